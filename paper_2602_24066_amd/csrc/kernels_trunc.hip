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

// Rows of a launch: (path, time chunk) pairs, or, with a window list (Section 5: signatures over windows), (path,
// window) pairs: window k is the path between the points win[2 k] and win[2 k + 1] (clamped to the path), at most
// max_len segments.  Every window of every path advances as a row of its own, read straight from the path.
__device__ __forceinline__ void row_segments(const WindowList& wl, int64_t row, int64_t P, int64_t C, int64_t Lc,
                                             int64_t& b, int64_t& seg0, int64_t& L)
{
    if (wl.win == nullptr) {
        b = row / C;
        seg0 = (row - b * C) * Lc;
        L = (P - 1 - seg0) < Lc ? (P - 1 - seg0) : Lc;
    } else {
        b = row / wl.K;
        const int64_t k = row - b * wl.K;
        int64_t l = wl.win[2 * k], r = wl.win[2 * k + 1];
        l = l < 0 ? 0 : (l > P - 1 ? P - 1 : l);
        r = r < l ? l : (r > P - 1 ? P - 1 : r);
        seg0 = l;
        L = r - l < wl.max_len ? r - l : wl.max_len;
    }
}

template <int D, int N, int K, int WQ, int T>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void trunc_mfma_fwd_kernel(const float* __restrict__ path,
                                                                                int64_t B, int64_t P, int64_t C, int64_t Lc,
                                                                                WindowList wl, float* __restrict__ coeffs)
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
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // the same in every lane: scalar registers
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + wib;
    if (wave >= B * C * (wl.win ? wl.K : 1) * G::WAVES) return;   // no barriers below: a whole wavefront may leave
    float (*E)[N][D] = E_all[wib];
    float (*Ec)[D][NC] = Ec_all[wib];
    // row = (path, chunk): chunk c of a path covers its segments [c Lc, min((c + 1) Lc, P - 1)) and is treated as
    // a path of its own whose signature goes to row `row` of coeffs (C = 1: the whole path); or (path, window)
    const int64_t row = wave / G::WAVES;
    int64_t b, seg0, L;
    row_segments(wl, row, P, C, Lc, b, seg0, L);
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
    const float* X = path + (b * P + seg0) * D;

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
            const int64_t jc = jj < L ? jj : (L > 0 ? L - 1 : 0);
            const int i = e % D;
            const float x1 = X[(jc + (L > 0 ? 1 : 0)) * D + i], x0 = X[jc * D + i];   // an empty window reads its own point
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

    float* out = coeffs + row * (int64_t)(level_start(D, N) + ipow(D, N));
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
hipError_t launch_trunc_mfma_fwd(const float* path, int64_t B, int64_t P, int64_t C, int64_t Lc, float* coeffs,
                                 hipStream_t stream, const WindowList& wl = WindowList())
{
    using G = MGeo<D, N, K, WQ>;
    constexpr int T = G::WIDE ? 8 : 16;          // d = 16: 32 KB of LDS per workgroup, so that three fit on a compute unit
    const int64_t waves = B * C * (wl.win ? wl.K : 1) * G::WAVES;
    const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    trunc_mfma_fwd_kernel<D, N, K, WQ, T><<<(unsigned)blocks, kWave * kWavesPerBlock, 0, stream>>>(path, B, P, C, Lc, wl, coeffs);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------------------
// Backward for units whose cascade has exactly two levels below the chain (K = N - 2): the slice level holds
// the words of length N - 1 and their children are the words of length N (leaves).
//
// Per segment j = L..1 (Section 4):
//   1. S_{0,t_{j-1}} = S_{0,t_j} (x) exp(-dX_j)  (Proposition 4.6): the forward update with -dX, chain on the
//      vector ALU, slice and leaves on the matrix cores.
//   2. the Horner accumulators A+ are recomputed from the reconstructed signature with +dX (chain: vector ALU,
//      slice: one matrix instruction per letter group).
//   3. adjoint of the update, bottom up.  For a word u with parent p, target offset t and c = dX^{(u_k)}/(t+1):
//         dLoss/d dX^{(u_k)} += gbar_u[t] * A+_p[t+1] / (t+1),   gbar_p[t+1] += c * gbar_u[t],
//         Abar_{j-1}(u) = sum_t gbar_u[t],                        gbar_u[0] = Abar_j(u),
//      which is Proposition 4.1 with the right factors S_{t_j,T} aggregated over all words sharing a prefix.
//      The adjoints of the leaves are constant (= grad_coeffs) and kept twice: in the layout of the parent word
//      vector ("node layout": lane = parent, one register per letter) for the contraction over letters, and in
//      the matrix cores' result layout ("child layout") for the contraction over parents, where every lane
//      accumulates the gradient of a single letter.  Parent values are brought into the child layout by a
//      matrix instruction with B = 1 (a broadcast inside each block).
// Gradient contributions are summed per wavefront in an LDS tile [T][D] with LDS atomics and flushed per tile
// with global atomics (several wavefronts work on one path).

__device__ __forceinline__ float dpp_quad(float v, int /*ctrl: compile-time*/ which)
{
    // which = 1: lanes (0,1)(2,3) swapped; which = 2: lanes (0,2)(1,3) swapped, inside each group of four
    const int x = __builtin_bit_cast(int, v);
    const int y = which == 1 ? __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true)
                             : __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true);
    return __builtin_bit_cast(float, y);
}

// M[r] in lane 4*blk + j is a contribution to the word of lane 4*blk + r; returns, in lane 4*blk + i, the sum
// over the four lanes of the block of M[i].
__device__ __forceinline__ float quad_transpose_reduce(const float (&M)[4], int lane)
{
    const bool o1 = (lane & 1) != 0, o2 = (lane & 2) != 0;
    const float keep0 = o1 ? M[1] : M[0], send0 = o1 ? M[0] : M[1];
    const float keep1 = o1 ? M[3] : M[2], send1 = o1 ? M[2] : M[3];
    const float u0 = keep0 + dpp_quad(send0, 1);
    const float u1 = keep1 + dpp_quad(send1, 1);
    const float keep = o2 ? u1 : u0, send = o2 ? u0 : u1;
    return keep + dpp_quad(send, 2);
}

__host__ __device__ constexpr int ilog2(int x)
{
    int r = 0;
    while ((1 << (r + 1)) <= x) ++r;
    return r;
}

__host__ __device__ constexpr int popcount6(int x)
{
    int r = 0;
    for (int bit = 0; bit < 6; ++bit) r += (x >> bit) & 1;
    return r;
}
// deposit the low bits of i into the lane-number bits that are NOT in keep / collect them back
__host__ __device__ constexpr int spread_bits(int keep, int i)
{
    int r = 0, src = 0;
    for (int bit = 0; bit < 6; ++bit)
        if (!((keep >> bit) & 1)) { r |= ((i >> src) & 1) << bit; ++src; }
    return r;
}
__device__ __forceinline__ int gather_bits(int keep, int lane)
{
    int r = 0, dst = 0;
#pragma unroll
    for (int bit = 0; bit < 6; ++bit)
        if (!((keep >> bit) & 1)) { r |= ((lane >> bit) & 1) << dst; ++dst; }
    return r;
}

// V[T][64]: one value per (segment, lane).  Lanes that agree on the lane-number bits in KEEP contribute to the same
// letter (my_letter, valid in every lane of the class).  Each class sums its values per segment and adds the
// result to gt[segment][letter]; the lanes of a class split the segments between them.
// The classes of a call carry different letters and the lanes of a class take different segments, so no two lanes of a
// call meet in one entry of gt, and the calls of a wavefront follow each other in order: a plain read-modify-write
// does (LDS floating-point atomics were measured at some ninety clocks each and cost the d = 16 backward kernel a
// sixth of its time).  ATOMIC = true is for a caller whose classes may share a letter.
template <int KEEP, int T, bool ATOMIC = false>
__device__ __forceinline__ void tile_reduce(const float* V, float* gt, int D, int lane, int my_letter)
{
    constexpr int NL = 1 << (6 - popcount6(KEEP));     // lanes per class
    const int m = gather_bits(KEEP, lane);
#pragma unroll
    for (int t0 = 0; t0 < T; t0 += NL) {
        const int tt = t0 + m;
        if (tt < T) {
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < NL; ++i) acc += V[tt * kWave + ((lane & KEEP) | spread_bits(KEEP, i))];
            if constexpr (ATOMIC) __hip_atomic_fetch_add(gt + tt * D + my_letter, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else gt[tt * D + my_letter] += acc;
        }
    }
}

// Values of other lanes without LDS traffic: DPP forms inside a row of 16 lanes (CTRL: 0x120 + n lane + n mod 16, 0x140 lane
// 15 - l, 0x141 lane 7 - l of the half row, 0xB1 / 0x4E lanes l ^ 1 / l ^ 2 of the quad), the swizzle network for an
// exclusive-or of the lane number below 32.  Every lane must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
template <int XOR_MASK>
__device__ __forceinline__ float swizzle_xor(float x)
{
    static_assert(XOR_MASK > 0 && XOR_MASK < 32, "the swizzle network works on groups of 32 lanes");
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), (XOR_MASK << 10) | 0x1f));
}
// The same exchange across rows with the swap instructions of gfx950 (vector ALU, no LDS round trip, no selects):
// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 of its second, v_permlane16_swap
// the odd rows of 16 lanes of the first with the even rows of the second.  After the swap the two registers hold, in
// every lane, this lane's and its partner's (lane ^ 32, lane ^ 16) value of the operand the lane keeps: `a` in the lower
// half / the even rows, `b` in the upper half / the odd rows.
__device__ __forceinline__ float fold_swap32(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float fold_swap16(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Four values per lane (v[s] belongs to segment s) summed over pairs of partner lanes, twice, each time keeping half of
// the segments: the lane ends up with the sum over four lanes for segment 2 hi + lo.  X1 / X2 fetch the partner's value;
// the partner of the first exchange differs in `hi`, the partner of the second agrees in `hi` and differs in `lo`.
template <class X1, class X2>
__device__ __forceinline__ float fold_four_segments(const float (&v)[4], bool hi, bool lo, X1 x1, X2 x2)
{
    const float k0 = hi ? v[2] : v[0], k1 = hi ? v[3] : v[1];
    const float s0 = hi ? v[0] : v[2], s1 = hi ? v[1] : v[3];
    const float a0 = k0 + x1(s0), a1 = k1 + x1(s1);
    return (lo ? a1 : a0) + x2(lo ? a0 : a1);
}

// One round of the same exchange on an array: v[0 .. N/2) <- the half of v this lane keeps (the upper one where `upper`)
// plus the other half of the partner lane, which keeps the opposite one.  Repeated with partners that agree in the bits
// used so far, the N values of every lane end up spread over the lanes, each summed over the lanes visited.
template <int N, class X>
__device__ __forceinline__ void fold_halves(float* v, bool upper, X partner)
{
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const float keep = upper ? v[i + N / 2] : v[i];
        const float send = upper ? v[i] : v[i + N / 2];
        v[i] = keep + partner(send);
    }
}

// chain letter k (0-based) of K: bit field of the lane number, or empty when the letter is the same in the whole wavefront
__host__ __device__ constexpr int chain_keep_mask(int LB, int K, int k)
{
    const int lo = LB * (K - 1 - k);
    return lo >= 6 ? 0 : ((((1 << LB) - 1) << lo) & 63);
}

template <int D, int K, int T, int KI, bool ATOMIC = false>
__device__ __forceinline__ void chain_tile_reduce(const float* Vsrc, float* gt, int lane, const int (&letter)[K])
{
    if constexpr (KI < K - 1) {
        tile_reduce<chain_keep_mask(ilog2(D), K, KI), T, ATOMIC>(Vsrc + KI * T * kWave, gt, D, lane, letter[KI]);
        chain_tile_reduce<D, K, T, KI + 1, ATOMIC>(Vsrc, gt, lane, letter);
    }
}

// Reconstruction check: after the walk back over a whole path the reconstructed signature is that of the empty path,
// whose coefficients of non-empty words are zero (Lemma 4.5, Proposition 4.6).  resid[b] receives the largest
// absolute value a wavefront still holds (non-negative floats order like their bit patterns).
__device__ __forceinline__ void report_residual(float m, float* resid, int64_t b)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) atomicMax((int*)resid + b, __float_as_int(m));
}

// LDS of one wavefront of the backward kernel for d = 16, in floats.  The leaf level (adjoints constant in time) is
// handled by time-batched matrix products over a tile of 16 segments, which need the slice-level values of the
// tile in LDS (HA).
template <int D, int N, int WQ, int T, int VG>
struct BwdLds {
    using G = MGeo<D, N, N - 2, WQ>;
    static_assert(G::WIDE, "sixteen letters: the leaves of a slice word fill a 16x16 matrix instruction");
    static_assert(T % VG == 0 && VG % 2 == 0, "the gradient sources are summed every VG segments");
    static constexpr int NC = (N + 3) / 4 * 4;
    static constexpr int NSV = WQ * 4;
    static constexpr int NSRC = 1 + WQ + (N - 2 - 1);
    static constexpr int SP = 68;                       // row stride of HA: 64 parents + 4 (16-byte aligned rows whose
                                                        // columns fall into different banks)
    // the table of scaled increments of a tile is the same for the wavefronts of a workgroup (they walk the same
    // row) and sits once at the start of LDS; the rest is private to a wavefront
    static constexpr int EC_FLOATS = T * D * NC;
    static constexpr int OFF_GT = 0;
    static constexpr int OFF_VB = OFF_GT + T * D;
    // the shapes for two workgroups per compute unit keep the gradient sources of VG = 4 segments in registers and sum
    // them over lanes with cross-lane moves; the other shapes park them in LDS (VB)
    static constexpr bool SOURCES_IN_REGISTERS = VG == 4 && T > VG && D == 16 && N == 4 && WQ == 1;
    static constexpr int OFF_HA = OFF_VB + (SOURCES_IN_REGISTERS ? 0 : NSRC * VG * kWave);
    static constexpr int PER_WAVE = OFF_HA + NSV * T * SP;
    static_assert(EC_FLOATS % 4 == 0 && OFF_VB % 4 == 0 && OFF_HA % 4 == 0 && PER_WAVE % 4 == 0,
                  "16-byte alignment of the LDS regions");
    static constexpr bool TWO_WORKGROUPS = SOURCES_IN_REGISTERS;   // per compute unit: registers held to half a SIMD's
    static constexpr size_t BYTES = ((size_t)EC_FLOATS + (size_t)kWavesPerBlock * PER_WAVE) * sizeof(float);
};

template <int D, int N, int WQ, int T, int VG>
__global__ __launch_bounds__(kWave * kWavesPerBlock, (BwdLds<D, N, WQ, T, VG>::TWO_WORKGROUPS ? 2 : 1)) void trunc_mfma_bwd_kernel(
    const float* __restrict__ path, const float* __restrict__ coeffs, const float* __restrict__ grad,
    const float* __restrict__ coeffs_last, const float* __restrict__ grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc,
    WindowList wl, float* gdx, float* resid)
{
    static_assert((D & (D - 1)) == 0, "the gradient reduction takes letters as bit fields of the lane number");
    constexpr int K = N - 2;
    using G = MGeo<D, N, K, WQ>;
    static_assert(G::WIDE, "sixteen letters; narrower alphabets take trunc_node_bwd_kernel");
    constexpr int NBS = G::NBS;                       // slice combinations: index t * WQ + g, t in {0, 1}
    constexpr int NC = (N + 3) / 4 * 4;
    constexpr int NSV = WQ * 4;                       // slice word vectors
    constexpr int NSRC0 = 1 + WQ;                     // sources before the earlier chain letters
    constexpr int LB = ilog2(D);
    using LY = BwdLds<D, N, WQ, T, VG>;
    static_assert(T <= 16 && T % 2 == 0, "the time-batched leaf products take up to 16 segments per matrix instruction");
    static_assert(T * D <= kWave * kWavesPerBlock, "one element of the increment tile per thread");
    static_assert(G::WAVES % kWavesPerBlock == 0, "the wavefronts of a workgroup walk the same row: they share the table of "
                                                  "increments and meet at its barriers");
    extern __shared__ v4f bwd_smem[];

    const int lane = threadIdx.x % kWave;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // the same in every lane: scalar registers
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + wib;
    if (wave >= B * C * (wl.win ? wl.K : 1) * G::WAVES) return;          // whole workgroups: the row count is a multiple
    float* const lds = (float*)bwd_smem + LY::EC_FLOATS + wib * LY::PER_WAVE;   // wave-private
    float (*Ec)[D][NC] = (float (*)[D][NC])bwd_smem;                    // Ec[segment][letter][t] = dX^{(letter)} / (t + 1), shared
    float* gt = lds + LY::OFF_GT;
    float* Vb = lds + LY::OFF_VB;
    float* HA = lds + LY::OFF_HA;                                       // [NSV][T][SP]
    constexpr int SP = LY::SP;
    constexpr int KS = D / 4;
    // row = (path, chunk): walks the segments [c Lc, min((c + 1) Lc, P - 1)) of path b backwards, starting from
    // row `row` of coeffs (signature up to the end of the chunk) and of grad (adjoint at the end of the chunk)
    const int64_t row = wave / G::WAVES;
    int64_t b, seg0, L;
    row_segments(wl, row, P, C, Lc, b, seg0, L);
    if (L <= 0) return;                                                  // an empty window: no gradient
    const int wip = (int)(wave % G::WAVES);
    const int slice = wip % G::NSL;
    const int p = (wip / G::NSL) * kWave + lane;
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const int g0 = slice * WQ;
    const float* X = path + (b * P + seg0) * D;
    const int64_t nW = level_start(D, N) + ipow(D, N);
    // rows of the last chunk of a path may live in arrays of their own ([B][|W|]: the caller's terminal signature
    // and gradient); the others in a [B][C][|W|] array of signatures and, then, a [B][C - 1][|W|] array of adjoints
    const bool in_last = coeffs_last != nullptr && row - b * C == C - 1;
    const float* cf = in_last ? coeffs_last + b * nW : coeffs + row * nW;
    const float* gr = in_last ? grad_last + b * nW : grad + (coeffs_last != nullptr ? row - b : row) * nW;

    int offS[NBS];
#pragma unroll
    for (int r = 0; r < NBS; ++r) {
        const int c = 4 * r + lane / 16;
        offS[r] = c < 2 * WQ ? (4 * (g0 + c % WQ) + (lane & 3)) * NC + c / WQ : 0;
    }

    // ---- state: terminal signature and adjoints
    float Sc[K], Ac[K];
    v4f S1[WQ], A1[WQ];
    // The coefficients of the leaves are never needed (their adjoints are the gradient itself).  Leaf adjoints
    // G[v][parent][letter] as A operands of the 16x16x4 matrix instruction (lane l supplies row l % 16, k = l / 16).
    // Ga: rows = parents 16 mb + l % 16, k = letters 4 ks + l / 16 (contraction over letters);
    // Gt: rows = letters l % 16, k = parents 4 ks + l / 16 (contraction over parents).
    float Ga[NSV][4][KS];
    float Gt[NSV][16];
    int phi = 0;
#pragma unroll
    for (int k = 1; k <= K; ++k) {
        phi = phi * D + letter[k - 1];
        const bool owner = (p % ipow(D, K - k) == 0) && slice == 0;
        Sc[k - 1] = cf[level_start(D, k) + phi];
        Ac[k - 1] = owner ? gr[level_start(D, k) + phi] : 0.0f;
    }
#pragma unroll
    for (int g = 0; g < WQ; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ph = __shfl(phi, (lane & ~3) + r) * D + 4 * (g0 + g) + (lane & 3);   // word of slice vector (g, r) in this lane
            S1[g][r] = cf[level_start(D, N - 1) + ph];
            A1[g][r] = gr[level_start(D, N - 1) + ph];
            const int v = g * 4 + r;
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    Ga[v][mb][ks] = gr[level_start(D, N) + __shfl(ph, 16 * mb + (lane & 15)) * D + 4 * ks + lane / 16];
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) {
                const int pw = __shfl(ph, 4 * ks + lane / 16);
                Gt[v][ks] = (lane & 15) < D ? gr[level_start(D, N) + pw * D + (lane & 15)] : 0.0f;
            }
        }

    // the workgroup loads a tile of increments together: thread e takes (segment e / D, letter e % D)
    float dxn;
    const int tile_e = (int)threadIdx.x < T * D ? (int)threadIdx.x : T * D - 1;
    auto fetch = [&](int64_t j0) {
        int64_t jj = j0 + tile_e / D;
        const bool ok = jj >= 0 && jj < L;
        jj = jj < 0 ? 0 : (jj < L ? jj : L - 1);
        const int i = tile_e % D;
        const float x1 = X[(jj + 1) * D + i], x0 = X[jj * D + i];
        dxn = ok ? x1 - x0 : 0.0f;
    };
    auto stage = [&]() {
        if ((int)threadIdx.x < T * D) {
#pragma unroll
            for (int t = 0; t < N; ++t) Ec[tile_e / D][tile_e % D][t] = dxn * inv1(t);
        }
    };
    const v4f zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const float one = 1.0f;

    // A segment is processed in two phases.  recon: steps 1 and 2 of the list above (they only depend on the
    // signature); adjoint: step 3 (depends on the adjoints and on what recon left in `Saved`).  The tile loop runs
    // recon one segment ahead of adjoint, so that the two dependent chains of a lone wavefront overlap.
    struct Saved {
        float ec[K][NC];
        float ap[K + 1][N + 2];
        v4f Gp[WQ];
        v4f Pb1, Pb2;
        float b0v[WQ];
    };
    auto recon = [&](int row, Saved& sv) {
        const float* Et = &Ec[row][0][0];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const float* src = &Ec[row][letter[k]][0];
#pragma unroll
            for (int t = 0; t <= N - (k + 1); ++t) sv.ec[k][t] = src[t];
        }
        float bs[NBS], nbs[NBS];
#pragma unroll
        for (int r = 0; r < NBS; ++r) { bs[r] = Et[offS[r]]; nbs[r] = -bs[r]; }
#pragma unroll
        for (int g = 0; g < WQ; ++g) sv.b0v[g] = Et[(4 * (g0 + g) + (lane & 3)) * NC];

        // 1. reconstruction with -dX
        float am[K + 1][N + 2];
#pragma unroll
        for (int t = 0; t < N + 2; ++t) am[0][t] = 1.0f;
#pragma unroll
        for (int k = 1; k <= K; ++k) {
#pragma unroll
            for (int t = 1; t <= N - k; ++t) am[k][t] = fmaf(-sv.ec[k - 1][t], am[k - 1][t + 1], Sc[k - 1]);
            Sc[k - 1] = fmaf(-sv.ec[k - 1][0], am[k - 1][1], Sc[k - 1]);
        }
#pragma unroll
        for (int g = 0; g < WQ; ++g) S1[g] = mfma4(am[K][1], nbs[g / 4], S1[g], g % 4);
        // 2. accumulators with +dX from the reconstructed signature
#pragma unroll
        for (int t = 0; t < N + 2; ++t) sv.ap[0][t] = 1.0f;
#pragma unroll
        for (int k = 1; k <= K; ++k)
#pragma unroll
            for (int t = 1; t <= N - k; ++t) sv.ap[k][t] = fmaf(sv.ec[k - 1][t], sv.ap[k - 1][t + 1], Sc[k - 1]);
#pragma unroll
        for (int g = 0; g < WQ; ++g) sv.Gp[g] = mfma4(sv.ap[K][2], bs[(WQ + g) / 4], S1[g], (WQ + g) % 4);
        // chain values A+_K[1], A+_K[2]/2 of the parent of every slice word, in the child layout
        sv.Pb1 = __builtin_amdgcn_mfma_f32_4x4x1f32(sv.ap[K][1], one, zero4, 0, 0, 0);
        sv.Pb2 = __builtin_amdgcn_mfma_f32_4x4x1f32(0.5f * sv.ap[K][2], one, zero4, 0, 0, 0);
    };

    struct Sources { float last, slice, first; };     // gradient sources of a segment: letter[K - 1], slice letter, letter[0]
    // A+ of parent p goes to slot (p % 4) * 16 + p / 4 of its row: the product over parents after the segment loop
    // reads parents 4 ks + lane / 16, ks = 0..15, which are then 16 consecutive floats.  (All lanes read their
    // gbar[1] from the row before any of them writes into it.)
    const int aplus_slot = (lane & 3) * 16 + (lane >> 2);
    auto adjoint = [&](int row, const Saved& sv, Sources& src) {
        // 3a. leaves: gbar[1] of the slice word was computed for the whole tile before the segment loop; its slot
        // takes A+_{N-1}[1] of the slice word for the product over parents after the loop
        v4f g1[WQ];
#pragma unroll
        for (int v = 0; v < NSV; ++v) {
            float* slots = HA + (v * T + row) * SP;
            g1[v / 4][v % 4] = slots[lane];
            slots[aplus_slot] = sv.Gp[v / 4][v % 4];
        }
        // 3b. slice words
        float gcs[WQ], M1[4], M2[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) M1[r] = M2[r] = 0.0f;
#pragma unroll
        for (int g = 0; g < WQ; ++g) {
            gcs[g] = 0.0f;
            const float b1v = 0.5f * sv.b0v[g];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float q0 = A1[g][r], q1 = g1[g][r];
                gcs[g] = fmaf(q0, sv.Pb1[r], gcs[g]);
                gcs[g] = fmaf(q1, sv.Pb2[r], gcs[g]);
                M1[r] = fmaf(sv.b0v[g], q0, M1[r]);
                M2[r] = fmaf(b1v, q1, M2[r]);
                A1[g][r] = q0 + q1;
            }
        }
        // 3c. chain
        float gb[K + 1][N + 2];
#pragma unroll
        for (int k = 0; k <= K; ++k)
#pragma unroll
            for (int t = 0; t < N + 2; ++t) gb[k][t] = 0.0f;
        gb[K][1] = quad_transpose_reduce(M1, lane);
        gb[K][2] = quad_transpose_reduce(M2, lane);
        float gck[K];
#pragma unroll
        for (int k = K; k >= 1; --k) {
            gb[k][0] = Ac[k - 1];
            float gc = 0.0f, asum = 0.0f;
#pragma unroll
            for (int t = 0; t <= N - k; ++t) {
                const float q = gb[k][t];
                asum += q;
                gc = fmaf(q * inv1(t), sv.ap[k - 1][t + 1], gc);
                gb[k - 1][t + 1] = fmaf(sv.ec[k - 1][t], q, gb[k - 1][t + 1]);
            }
            Ac[k - 1] = asum;
            gck[k - 1] = gc;
        }
        // 4. gradient contributions of this segment: every lane parks its values in private LDS slots
        //    Vb[source][segment][lane]; they are summed over lanes once per tile (tile_reduce), which keeps
        //    dependent cross-lane chains out of the segment loop.
        if constexpr (LY::SOURCES_IN_REGISTERS) {
            src.last = gck[K - 1];
            src.slice = gcs[0];
            src.first = gck[0];
        } else {
            float* vb = Vb + (row % VG) * kWave + lane;
            vb[0] = gck[K - 1];                                       // source 0: letters = lane bits [0, LB)
#pragma unroll
            for (int g = 0; g < WQ; ++g) vb[(1 + g) * VG * kWave] = gcs[g];   // sources 1..WQ: letters 4 (g0 + g) + lane % 4
#pragma unroll
            for (int k = 0; k < K - 1; ++k) vb[(NSRC0 + k) * VG * kWave] = gck[k];   // earlier chain letters
        }
    };
    // The same sums with the sources of four segments in registers (d = 16, depth 4: letter[1] = lane bits 0..3, the
    // slice letter = 4 g0 + lane bits 0..1, letter[0] = lane bits 4..5 of this wavefront's 64 parents).  Each source
    // is folded over the lane bits its letter does not depend on; two of those bits select the segment a lane ends up
    // with, so the four segments cost little more than one.
    auto reduce_registers = [&](int first, const float (&last)[4], const float (&slice)[4], const float (&chain0)[4]) {
        float* gtv = gt + first * D;
        // letter[1]: classes of the four lanes that differ in bits 4, 5; every lane ends with one (segment, letter)
        const float r0 = fold_swap16(fold_swap32(last[0], last[2]), fold_swap32(last[1], last[3]));
        gtv[(lane >> 4) * D + letter[K - 1]] += r0;
        // slice letter: classes of sixteen lanes that differ in bits 2..5 (inside a row: lanes l, l + 4, l + 8, l + 12)
        float r1 = fold_swap16(fold_swap32(slice[0], slice[2]), fold_swap32(slice[1], slice[3]));
        r1 += dpp_lane<0x128>(r1);
        r1 += dpp_lane<0x124>(r1);
        if ((lane & 12) == 0) gtv[(lane >> 4) * D + 4 * g0 + (lane & 3)] += r1;
        // letter[0]: classes of the sixteen lanes of a row
        float r2 = fold_four_segments(chain0, (lane & 8) != 0, (lane & 4) != 0, [](float x) { return dpp_lane<0x140>(x); },
                                      [](float x) { return dpp_lane<0x141>(x); });
        r2 += dpp_lane<0xB1>(r2);
        r2 += dpp_lane<0x4E>(r2);
        if ((lane & 3) == 0) gtv[((lane >> 2) & 3) * D + letter[0]] += r2;
    };

    // the sources of the VG segments from `first` on, summed over the lanes into the gradient tile
    auto reduce_sources = [&](int first) {
        wave_lds_fence();
        float* gtv = gt + first * D;
        // (the lanes of a class take different segments and the classes of a source different letters: no two lanes of
        // a call meet in one entry, so plain read-modify-writes do; LDS atomics cost some ninety clocks each)
        tile_reduce<(1 << LB) - 1, VG, false>(Vb, gtv, D, lane, letter[K - 1]);
#pragma unroll
        for (int g = 0; g < WQ; ++g)
            tile_reduce<3, VG, false>(Vb + (1 + g) * VG * kWave, gtv, D, lane, 4 * (g0 + g) + (lane & 3));
        chain_tile_reduce<D, K, VG, 0, false>(Vb + NSRC0 * VG * kWave, gtv, lane, letter);
        wave_lds_fence();
    };


    const int64_t ntiles = (L + T - 1) / T;
    for (int e = lane; e < T * D; e += kWave) gt[e] = 0.0f;
    fetch((ntiles - 1) * T);
    for (int64_t n = ntiles - 1; n >= 0; --n) {
        __syncthreads();                               // every wavefront is done with the table of the tile before
        stage();
        __syncthreads();
        fetch((n - 1) * T);                            // n = 0: out of range, zeros
        {
            // gbar[1](slice word p, segment s) = sum_j dX_s^{(j)} G[p][j] for the 16 segments of the tile:
            // [64 parents x D letters] . [D letters x 16 segments] per slice vector; the result (row = parent
            // 4 (l / 16) + r of block mb, column = segment l % 16) goes to HA[v][segment][parent]
            // (a tile of 8 segments fills half of the 16 columns; the other lanes compute on a copy and store nothing)
            const int col = (lane & 15) % T;
            const bool col_ok = (lane & 15) < T;
            float Bx[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) Bx[ks] = Ec[col][4 * ks + lane / 16][0];
#pragma unroll
            for (int v = 0; v < NSV; ++v)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) {
                    v4f acc = zero4;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Ga[v][mb][ks], Bx[ks], acc, 0, 0, 0);
                    if (T == 16 || col_ok) *(v4f*)(HA + (v * T + col) * SP + 16 * mb + 4 * (lane / 16)) = acc;
                }
            wave_lds_fence();
        }
        {
            static_assert(T % 2 == 0, "the segment loop is unrolled by two");
            if constexpr (T == 16 && !LY::TWO_WORKGROUPS) {
                // a lone wavefront per SIMD: recon runs one segment ahead of adjoint so that their chains overlap
                Saved SA, SB;
                Sources unused;
                recon(T - 1, SA);
#pragma unroll 1
                for (int tt = T - 1; tt >= 3; tt -= 2) {
                    recon(tt - 1, SB);
                    adjoint(tt, SA, unused);
                    recon(tt - 2, SA);
                    adjoint(tt - 1, SB, unused);
                    if constexpr (VG < T) {
                        if ((tt - 1) % VG == 0) reduce_sources(tt - 1);
                    }
                }
                recon(0, SB);
                adjoint(1, SA, unused);
                adjoint(0, SB, unused);
            } else if constexpr (LY::SOURCES_IN_REGISTERS) {
#pragma unroll 1
                for (int t0 = T - VG; t0 >= 0; t0 -= VG) {
                    float last[VG], slice[VG], chain0[VG];
#pragma unroll
                    for (int i = VG - 1; i >= 0; --i) {
                        Saved SA;
                        Sources src;
                        recon(t0 + i, SA);
                        adjoint(t0 + i, SA, src);
                        last[i] = src.last;
                        slice[i] = src.slice;
                        chain0[i] = src.first;
                    }
                    reduce_registers(t0, last, slice, chain0);
                }
            } else {
                // two wavefronts per SIMD hide each other's latencies; one set of saved values keeps the registers
                // within half a SIMD's
#pragma unroll 1
                for (int tt = T - 1; tt >= 0; --tt) {
                    Saved SA;
                    Sources unused;
                    recon(tt, SA);
                    adjoint(tt, SA, unused);
                    if constexpr (VG < T) {
                        if (tt % VG == 0 && tt > 0) reduce_sources(tt);
                    }
                }
            }
        }
        wave_lds_fence();
        {
            // dLoss/d dX_s^{(j)} += sum_p G[p][j] A+(p, s): [D letters x 64 parents] . [64 parents x 16 segments] per
            // slice vector; row = letter 4 (l / 16) + r, column = segment l % 16
            const int col = (lane & 15) % T;
            v4f acc[4] = {zero4, zero4, zero4, zero4};
#pragma unroll
            for (int v = 0; v < NSV; ++v) {
                const v4f* bv = (const v4f*)(HA + (v * T + col) * SP + 16 * (lane / 16));
#pragma unroll
                for (int kq = 0; kq < 4; ++kq) {
                    const v4f b4 = bv[kq];
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        acc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(Gt[v][4 * kq + r], b4[r], acc[r], 0, 0, 0);
                }
            }
            const v4f sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
            if (4 * (lane / 16) < D && (T == 16 || (lane & 15) < T)) {
                v4f* dst = (v4f*)(gt + col * D + 4 * (lane / 16));
                *dst = *dst + sum;
            }
            wave_lds_fence();
        }
        if constexpr (!LY::SOURCES_IN_REGISTERS) reduce_sources(0);   // the last VG segments walked (all of them where VG = T)
        // flush: (segment, letter) is contiguous in gdx
        for (int e = lane; e < T * D; e += kWave) {
            const int64_t s = n * T + e / D;
            if (s < L) unsafeAtomicAdd(gdx + (b * (P - 1) + seg0 + n * T) * D + e, gt[e]);
            gt[e] = 0.0f;
        }
    }
    if (resid != nullptr && seg0 == 0) {
        float m = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k) m = fmaxf(m, fabsf(Sc[k]));
#pragma unroll
        for (int g = 0; g < WQ; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fmaxf(m, fabsf(S1[g][r]));
        report_residual(m, resid, b);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Backward with one wavefront per row for d = 4: a lane holds a word of length N - 3 (64 of them) and, in
// registers, its D children of length N - 2 ("tails", letter = register index, the same in every lane) with the
// D children of each ("slice words") and the gradients of the D leaves below each of those.  Everything below a
// tail is in the tail's lane and every letter there is the same in all lanes, so the two lower levels are plain
// multiply-adds with lane-uniform increments: the backward walk never reconstructs the leaf coefficients, and with
// D values per tail the slice level gains nothing from the matrix cores (an earlier form that kept it in the
// lane layout of trunc_mfma_bwd_kernel paid for transposes between the two layouts and ran 15 % slower).  Compared
// with four wavefronts per row that each hold one tail per lane, the chain above the tails is computed once
// instead of four times; rows are (path, time chunk) pairs, so the launcher cuts short batches into chunks to fill
// the chip.  No other wavefront writes the gradient of this row's segments: the tile is flushed with plain stores.
// CW = 0: rows are (path, chunk) pairs whose start signature and adjoint come from global arrays; every wavefront
// of a workgroup is an independent row.  CW = 2, 4 or 8 ("fused"): a workgroup is one path and its CW wavefronts are
// the CW chunks of it; the chunk signatures, their products and the adjoints at the chunk boundaries are formed inside
// the kernel and exchanged through LDS, so that nothing but path, terminal signature and gradient is read from HBM.
template <int D, int N, int T, int CW>
struct TailsLds {
    static constexpr int KL = N - 3;
    static constexpr int NC = (N + 3) / 4 * 4;
    static constexpr int NWV = CW ? CW : kWavesPerBlock;                     // wavefronts per workgroup
    // sources of gradient values: one per letter for tails, slice words and leaves (the same letter in every lane),
    // one per chain letter
    static constexpr int NSRC = D + KL;
    static constexpr int W = level_start(D, N) + ipow(D, N);
    // the chunk signatures and their products are kept up to length N - 1: the backward walk never reads the
    // coefficients of the longest words, and their adjoints are the gradient itself
    static constexpr int W1 = level_start(D, N);
    // scaled increments Ec of one wavefront, and for the chain rule the increment gradients of the first and of the
    // last segment of the row (2 D floats) and of the tile walked before (T D floats)
    static constexpr int TILE = T * D * NC + 2 * D + T * D;
    static constexpr int OFF_CG = T * D * NC;
    static constexpr int RED = T * D + NSRC * T * kWave;                     // gt, Vb of one wavefront
    // fused: area A holds first the signature buffers and a copy of the gradient row of the path, later the
    // reduction regions
    static constexpr int NBUF = CW > 2 ? 3 * CW - 4 : CW;                   // chunk signatures and running products
    static constexpr int BUFS = NBUF * W1 + W;
    static constexpr int AREA_A = CW ? (BUFS > NWV * RED ? BUFS : NWV * RED) : 0;
    // fused: the tiles come first (their addresses then fit the offset field of the LDS instructions), area A next
    static constexpr int OFF_A = CW ? NWV * TILE : 0;
    static constexpr int OFF_G = OFF_A + NBUF * W1;                           // fused: the gradient row of the path
    static constexpr int OFF_XY = OFF_A + AREA_A;     // fused: first / last segment gradients of the CW chunks
    static constexpr int TOTAL = CW ? OFF_XY + CW * 2 * D : NWV * (TILE + RED);
    static_assert(TILE % 4 == 0 && RED % 4 == 0 && AREA_A % 4 == 0 && W % 4 == 0 && W1 % 4 == 0, "16-byte alignment");
    static constexpr size_t BYTES = (size_t)TOTAL * sizeof(float);
    __device__ static float* tile(float* base, int wib) { return base + (CW ? wib * TILE : wib * (TILE + RED)); }
    __device__ static float* red(float* base, int wib) { return base + (CW ? OFF_A + wib * RED : wib * (TILE + RED) + TILE); }
};

// V[NS][T][64]: source s holds, for every segment, one value per lane, and all 64 lanes contribute to letter s.
// Lane s T + tt sums the row (s, tt) and adds it to gt[tt][first_letter + s].
template <int NS, int T>
__device__ __forceinline__ void tile_reduce_uniform(const float* V, float* gt, int D, int lane, int first_letter)
{
    static_assert(NS * T <= kWave, "one lane per (source, segment)");
    if (lane < NS * T) {
        // the rows lie 256 bytes apart: every lane starts at another 16-byte piece of its row, or all of them would
        // meet in the same four banks
        const v4f* row = (const v4f*)(V + lane * kWave);
        v4f acc = row[lane & 15];
#pragma unroll
        for (int i = 1; i < kWave / 4; ++i) acc += row[(i + lane) & 15];
        gt[(lane % T) * D + first_letter + lane / T] += (acc[0] + acc[1]) + (acc[2] + acc[3]);
    }
}

// sources KI .. KE - 1: the chain letters before the last one
template <int D, int KL, int T, int KI, int KE>
__device__ __forceinline__ void lane_chain_tile_reduce(const float* Vsrc, float* gt, int lane, const int (&letter)[KL])
{
    if constexpr (KI < KE) {
        tile_reduce<chain_keep_mask(ilog2(D), KL, KI), T>(Vsrc + KI * T * kWave, gt, D, lane, letter[KI]);
        lane_chain_tile_reduce<D, KL, T, KI + 1, KE>(Vsrc, gt, lane, letter);
    }
}

// out = a (x) b for signatures in LDS (canonical order), by nthreads threads; four consecutive words of a level
// share all prefixes and have contiguous suffixes (D = 4: one quad per parent).
template <int D, int N>
__device__ __forceinline__ void lds_tensor_product(const float* a, const float* b, float* out, int tid, int nthreads)
{
    constexpr int LB = ilog2(D);
#pragma unroll
    for (int n = 1; n <= N; ++n) {
        const int ls_n = level_start(D, n);
        const int quads = ipow(D, n) / 4;
        for (int qd = tid; qd < quads; qd += nthreads) {
            const int i = 4 * qd;
            v4f acc = *(const v4f*)(a + ls_n + i) + *(const v4f*)(b + ls_n + i);
#pragma unroll
            for (int k = 1; k < n; ++k) {
                const int sh = LB * (n - k);
                acc += a[level_start(D, k) + (i >> sh)] * *(const v4f*)(b + level_start(D, n - k) + (i & ((1 << sh) - 1)));
            }
            *(v4f*)(out + ls_n + i) = acc;
        }
    }
}
// coefficient of the word (length n, index i) of a (x) b
template <int D, int N>
__device__ __forceinline__ float word_product(const float* a, const float* b, int n, int i)
{
    constexpr int LB = ilog2(D);
    float acc = a[level_start(D, n) + i] + b[level_start(D, n) + i];
#pragma unroll
    for (int k = 1; k < N; ++k)
        if (k < n) {
            const int sh = LB * (n - k);
            acc = fmaf(a[level_start(D, k) + (i >> sh)], b[level_start(D, n - k) + (i & ((1 << sh) - 1))], acc);
        }
    return acc;
}
// adjoint of the word u (length n, index i) at a chunk boundary: g(u) + sum_{m >= 1} sum_{|v| = m} g(u v) q(v).
// `share` lanes (a power of two, consecutive, all holding the same u) split the sums; `sub` is the lane's rank.
// rot (a multiple of four, the same in the lanes of one u) rotates the order in which a lane walks its v, so that
// lanes whose words lie a power of two apart do not meet in one LDS bank.
template <int D, int N>
__device__ __forceinline__ float word_contract(const float* g, const float* q, int n, int i, int sub, int share, int rot)
{
    static_assert(D % 4 == 0, "the words u v of one u are read four at a time");
    constexpr int LB = ilog2(D);
    v4f acc4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int m = 1; m < N; ++m)
        if (m <= N - n) {
            const int cnt = 1 << (LB * m);
            const float* src = g + level_start(D, n + m) + (i << (LB * m));
            const float* qv = q + level_start(D, m);
            for (int v = 4 * sub; v < cnt; v += 4 * share) {
                const int vr = (v + rot) & (cnt - 1);
                acc4 += *(const v4f*)(src + vr) * *(const v4f*)(qv + vr);
            }
        }
    float acc = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
    for (int off = share >> 1; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    return g[level_start(D, n) + i] + acc;
}

template <int D, int N, int T, int CW, bool POINTS>
__global__ __launch_bounds__(kWave * (CW ? CW : kWavesPerBlock)) void trunc_tails_bwd_kernel(
    const float* __restrict__ path, const float* __restrict__ coeffs, const float* __restrict__ grad, int64_t B,
    int64_t P, int64_t C, int64_t Lc, WindowList wl, float* __restrict__ out)
{
    // POINTS (fused, or rows that are whole paths): the chain rule dX_j = X_{j+1} - X_j is applied here and out
    // receives the gradient with respect to the points [B, P, d]; otherwise the increment gradients [B, P - 1, d].
    static_assert(POINTS || CW == 0, "the fused form writes the gradient with respect to the points");
    float* const grad_path = out;
    float* const gdx = out;
    static_assert(D == 4, "one group of four letters");
    constexpr int K = N - 2;                          // length of the tail words
    constexpr int KL = K - 1;                         // letters held per lane
    static_assert(ipow(D, KL) == kWave, "64 words of length N - 3, one per lane");
    constexpr int NC = (N + 3) / 4 * 4;
    constexpr int EPL = (T * D + kWave - 1) / kWave;
    using LY = TailsLds<D, N, T, CW>;
    constexpr int TW = D;                             // tails per lane
    extern __shared__ v4f bwd_smem[];

    const int lane = threadIdx.x % kWave;
    // the same in every lane: said so, the row number and what follows from it (path, first segment, length, base
    // addresses) stay in scalar registers
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cib = wib;                              // fused: chunk of the workgroup's path
    const int64_t row = CW ? (int64_t)blockIdx.x * C + cib : (int64_t)blockIdx.x * kWavesPerBlock + wib;
    if constexpr (CW == 0) {
        if (row >= B * C * (wl.win ? wl.K : 1)) return;   // no workgroup barriers in this mode
    }
    float* const smem = (float*)bwd_smem;
    float (*Ec)[D][NC] = (float (*)[D][NC])(LY::tile(smem, wib));         // wave-private
    float* const cg = LY::tile(smem, wib) + LY::OFF_CG;                   // chain rule, see the flush below
    float* const pg = cg + 2 * D;
    float* gt = LY::red(smem, wib);                                       // fused: valid after the signature buffers
    float* Vb = gt + T * D;                                               // are dead
    int64_t b, seg0, L;
    row_segments(wl, row, P, C, Lc, b, seg0, L);      // (a window list comes with CW = 0 and without POINTS only)
    if constexpr (CW == 0) {
        if (L <= 0) return;                           // an empty window: no gradient
    }
    int letter[KL];
    {
        int q = lane;
#pragma unroll
        for (int k = KL - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + (b * P + seg0) * D;
    const int64_t nW = level_start(D, N) + ipow(D, N);
    // CW = 0: row arrays; fused: the terminal signature and the gradient of the path
    const float* cf = coeffs + (CW ? b : row) * nW;
    const float* gr = grad + (CW ? b : row) * nW;

    // ---- state
    float Sc[KL], Ac[KL];                  // per-lane chain: signature and adjoint (adjoint only in the owning lane)
    float St[TW], At[TW];                  // tails
    v4f S1[TW], A1[TW];                    // slice level: the D children of every tail
    float An[TW][D][D];                    // adjoints of the D leaves below every slice word, constant: the gradient;
                                           // the coefficients of the leaves are never needed

    float dxn[EPL];
    auto fetch = [&](int64_t j0) {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = (lane + q * kWave) < T * D ? lane + q * kWave : T * D - 1;
            int64_t jj = j0 + e / D;
            const bool ok = jj >= 0 && jj < L;
            jj = jj < 0 ? 0 : (jj < L ? jj : L - 1);
            const int i = e % D;
            const float x1 = X[(jj + 1) * D + i], x0 = X[jj * D + i];
            dxn[q] = ok ? x1 - x0 : 0.0f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = lane + q * kWave;
            if (e < T * D) {
#pragma unroll
                for (int t = 0; t < N; ++t) {
                    const float v = dxn[q] * inv1(t);
                    Ec[e / D][e % D][t] = v;
                }
            }
        }
    };

    // ---- initial state.  sig(n, i): coefficient of the word (length n, index i) the row starts from;
    // adj(n, i, sub, share): its adjoint (length < N), where `share` consecutive lanes hold the same word.
    auto load_signature = [&](auto&& sig) {
        int phi = 0;
#pragma unroll
        for (int k = 1; k <= KL; ++k) {
            phi = phi * D + letter[k - 1];
            Sc[k - 1] = sig(k, phi);
        }
#pragma unroll
        for (int ii = 0; ii < TW; ++ii) {
            const int i = ii;
            St[ii] = sig(K, lane * D + i);
#pragma unroll
            for (int j = 0; j < D; ++j) S1[ii][j] = sig(N - 1, (lane * D + i) * D + j);
        }
    };
    auto load_adjoint = [&](auto&& adj) {
        int phi = 0;
#pragma unroll
        for (int k = 1; k <= KL; ++k) {
            phi = phi * D + letter[k - 1];
            const int share = ipow(D, KL - k);                    // lanes holding this word
            const float v = adj(k, phi, lane % share, share);
            Ac[k - 1] = lane % share == 0 ? v : 0.0f;             // the adjoint lives in the owning lane only
        }
#pragma unroll
        for (int ii = 0; ii < TW; ++ii) {
            const int i = ii;
            At[ii] = adj(K, lane * D + i, 0, 1);
#pragma unroll
            for (int j = 0; j < D; ++j) A1[ii][j] = adj(N - 1, (lane * D + i) * D + j, 0, 1);
        }
    };
    // leaf adjoints are the gradient itself at every chunk boundary
#pragma unroll
    for (int ii = 0; ii < TW; ++ii)
#pragma unroll
        for (int j = 0; j < D; ++j)
#pragma unroll
            for (int jj = 0; jj < D; ++jj) An[ii][j][jj] = gr[level_start(D, N) + ((lane * D + ii) * D + j) * D + jj];

    if constexpr (CW == 0) {
        load_signature([&](int n, int i) { return cf[level_start(D, n) + i]; });
        load_adjoint([&](int n, int i, int, int) { return gr[level_start(D, n) + i]; });
    } else {
        constexpr int W = LY::W1;                      // words of length < N
        float* const SB = smem + LY::OFF_A;            // SB[c] = signature of chunk c
        float* const GB = smem + LY::OFF_G;            // the gradient row, read many times by the boundary adjoints
        for (int o = 4 * (int)threadIdx.x; o < LY::W; o += 4 * LY::NWV * kWave) *(v4f*)(GB + o) = *(const v4f*)(gr + o);
        // phase 1: signature of the own chunk, S <- S (x) exp(dX) segment by segment from the identity
        load_signature([&](int, int) { return 0.0f; });
        {
            const int64_t nt = (L + T - 1) / T;
            fetch(0);
            for (int64_t n = 0; n < nt; ++n) {
                wave_lds_fence();
                stage();
                wave_lds_fence();
                fetch((n + 1) * T);                    // beyond the chunk: zeros
#pragma unroll 2
                for (int tt = 0; tt < T; ++tt) {
                    float a[KL + 1][N + 2];
#pragma unroll
                    for (int t = 0; t < N + 2; ++t) a[0][t] = 1.0f;
#pragma unroll
                    for (int k = 1; k <= KL; ++k) {
                        const float* src = &Ec[tt][letter[k - 1]][0];
#pragma unroll
                        for (int t = 1; t <= N - k; ++t) a[k][t] = fmaf(src[t], a[k - 1][t + 1], Sc[k - 1]);
                        Sc[k - 1] = fmaf(src[0], a[k - 1][1], Sc[k - 1]);
                    }
#pragma unroll
                    for (int ii = 0; ii < TW; ++ii) {
                        const float* et = &Ec[tt][ii][0];
                        const float a1 = fmaf(et[1], a[KL][2], St[ii]);
                        St[ii] = fmaf(et[0], a[KL][1], St[ii]);
#pragma unroll
                        for (int j = 0; j < D; ++j) S1[ii][j] = fmaf(Ec[tt][j][0], a1, S1[ii][j]);
                    }
                }
            }
        }
        {   // publish it in canonical order
            float* out = SB + cib * W;
            int phi = 0;
#pragma unroll
            for (int k = 1; k <= KL; ++k) {
                phi = phi * D + letter[k - 1];
                if (lane % ipow(D, KL - k) == 0) out[level_start(D, k) + phi] = Sc[k - 1];
            }
#pragma unroll
            for (int ii = 0; ii < TW; ++ii) {
                const int i = ii;
                out[level_start(D, K) + lane * D + i] = St[ii];
                *(v4f*)(out + level_start(D, N - 1) + (lane * D + i) * D) = S1[ii];
            }
        }
        __syncthreads();
        // phase 2: what every chunk starts from.  With the chunks numbered from 0: E_k = S_0 (x) .. (x) S_k, the
        // signature at the end of chunk k, and Q_k = S_{k+1} (x) .. (x) S_{CW-1}, what follows it.  Both are running
        // products, CW - 2 rounds of two products each (one per half of the workgroup); E_0 = S_0 is in the
        // registers of chunk 0, E_{CW-1} is the terminal signature, Q_{CW-2} = S_{CW-1}.
        float* const EB = SB + CW * W;                 // EB[k - 1] = E_k, k = 1 .. CW - 2
        float* const QB = EB + (CW - 2) * W;           // QB[k] = Q_k, k = 0 .. CW - 3
        if constexpr (CW > 2) {
            constexpr int NT = LY::NWV * kWave / 2;
            const bool upper = (int)threadIdx.x >= NT;
            const int tid = (int)threadIdx.x - (upper ? NT : 0);
#pragma unroll 1
            for (int j = 1; j <= CW - 2; ++j) {
                if (!upper)
                    lds_tensor_product<D, N - 1>(j == 1 ? SB : EB + (j - 2) * W, SB + j * W, EB + (j - 1) * W, tid, NT);
                else
                    lds_tensor_product<D, N - 1>(SB + (CW - 1 - j) * W, j == 1 ? SB + (CW - 1) * W : QB + (CW - 1 - j) * W,
                                                 QB + (CW - 2 - j) * W, tid, NT);
                __syncthreads();
            }
            if (cib >= 1 && cib <= CW - 2) {
                const float* e = EB + (cib - 1) * W;
                load_signature([&](int n, int i) { return e[level_start(D, n) + i]; });
            }
        }
        const float* qbuf = cib == CW - 2 ? SB + (CW - 1) * W : QB + cib * W;   // Q of the own chunk (not for the last)
        if (cib == CW - 1) {
            load_signature([&](int n, int i) { return cf[level_start(D, n) + i]; });                // terminal signature
            load_adjoint([&](int n, int i, int, int) { return gr[level_start(D, n) + i]; });
        } else {
            load_adjoint([&](int n, int i, int sub, int share) {
                return word_contract<D, N>(GB, qbuf, n, i, sub, share, 4 * (lane / share));
            });
        }
        __syncthreads();                               // the buffers are dead: their space takes gt / Vb from here on
    }

    auto step = [&](int row_t) {
        float ec[KL][NC];
#pragma unroll
        for (int k = 0; k < KL; ++k) {
            const float* src = &Ec[row_t][letter[k]][0];
#pragma unroll
            for (int t = 0; t <= N - (k + 1); ++t) ec[k][t] = src[t];
        }
        float eu[D][3];                               // dX^{(j)} / (t + 1), t = 0..2: the same in every lane
#pragma unroll
        for (int j = 0; j < D; ++j)
#pragma unroll
            for (int t = 0; t < 3; ++t) eu[j][t] = Ec[row_t][j][t];

        // 1. reconstruction with -dX, 2. accumulators with +dX (per-lane chain)
        float am[KL + 1][N + 2], ap[KL + 1][N + 2];
#pragma unroll
        for (int t = 0; t < N + 2; ++t) am[0][t] = ap[0][t] = 1.0f;
#pragma unroll
        for (int k = 1; k <= KL; ++k) {
#pragma unroll
            for (int t = 1; t <= N - k; ++t) am[k][t] = fmaf(-ec[k - 1][t], am[k - 1][t + 1], Sc[k - 1]);
            Sc[k - 1] = fmaf(-ec[k - 1][0], am[k - 1][1], Sc[k - 1]);
#pragma unroll
            for (int t = 1; t <= N - k; ++t) ap[k][t] = fmaf(ec[k - 1][t], ap[k - 1][t + 1], Sc[k - 1]);
        }
        float gbL[4] = {0.0f, 0.0f, 0.0f, 0.0f};      // gbar of the lane's word from its tails, t = 1..3
        float y[D];                                   // gradient of letter j from tails, slice words and leaves
#pragma unroll
        for (int j = 0; j < D; ++j) y[j] = 0.0f;
        float* vb = Vb + row_t * kWave + lane;
        // Everything below a tail lives in the tail's lane and every letter is the same in all lanes, so the two
        // levels are plain multiply-adds with lane-uniform increments (the matrix cores bring nothing here: the
        // leaf coefficients are not reconstructed, and the slice level is D values per tail).
#pragma unroll
        for (int i = 0; i < TW; ++i) {
            // tail i and its children: reconstruction, then the accumulators
            const float am1 = fmaf(-eu[i][1], am[KL][2], St[i]);
            St[i] = fmaf(-eu[i][0], am[KL][1], St[i]);
            const float ap1 = fmaf(eu[i][1], ap[KL][2], St[i]);
            const float ap2 = fmaf(eu[i][2], ap[KL][3], St[i]);
            const float hp2 = 0.5f * ap2;
            const float g0 = At[i];
            float g1 = 0.0f, g2 = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) {
                S1[i][j] = fmaf(-eu[j][0], am1, S1[i][j]);
                const float Gp = fmaf(eu[j][1], ap2, S1[i][j]);               // A+[1] of the slice word
                float h = 0.0f;                                                // its gbar[1], from the leaves
#pragma unroll
                for (int jj = 0; jj < D; ++jj) {
                    h = fmaf(eu[jj][0], An[i][j][jj], h);
                    y[jj] = fmaf(An[i][j][jj], Gp, y[jj]);                     // leaf letter jj
                }
                const float q0 = A1[i][j];
                A1[i][j] = q0 + h;
                y[j] = fmaf(q0, ap1, y[j]);                                    // slice letter j
                y[j] = fmaf(h, hp2, y[j]);
                g1 = fmaf(eu[j][0], q0, g1);                                   // what the slice word pushes up
                g2 = fmaf(eu[j][1], h, g2);
            }
            // the tail word itself: gbar[0] = its adjoint, gbar[1], gbar[2] pushed up from its children
            At[i] = g0 + g1 + g2;
            float gct = g0 * ap[KL][1];
            gct = fmaf(g1 * inv1(1), ap[KL][2], gct);
            gct = fmaf(g2 * inv1(2), ap[KL][3], gct);
            y[i] += gct;
            gbL[1] = fmaf(eu[i][0], g0, gbL[1]);
            gbL[2] = fmaf(eu[i][1], g1, gbL[2]);
            gbL[3] = fmaf(eu[i][2], g2, gbL[3]);
        }
        // 3d. per-lane chain.  The scaled increments of the chain letters are read from LDS a second time (through
        // an opaque copy of the letter, so that the two reads are not merged): keeping them in registers across the
        // tails would cost the registers that let two wavefronts share a SIMD.
        float gb[KL + 1][N + 2];
#pragma unroll
        for (int k = 0; k <= KL; ++k)
#pragma unroll
            for (int t = 0; t < N + 2; ++t) gb[k][t] = 0.0f;
#pragma unroll
        for (int t = 1; t <= 3; ++t) gb[KL][t] = gbL[t];
#pragma unroll
        for (int k = KL; k >= 1; --k) {
            int letter_again = letter[k - 1];
            asm volatile("" : "+v"(letter_again));
            const float* ec2 = &Ec[row_t][letter_again][0];
            gb[k][0] = Ac[k - 1];
            float gc = 0.0f, asum = 0.0f;
#pragma unroll
            for (int t = 0; t <= N - k; ++t) {
                const float q = gb[k][t];
                asum += q;
                gc = fmaf(q * inv1(t), ap[k - 1][t + 1], gc);
                if (k > 1) gb[k - 1][t + 1] = fmaf(ec2[t], q, gb[k - 1][t + 1]);
            }
            Ac[k - 1] = asum;
            vb[(D + (k - 1)) * T * kWave] = gc;                               // letter[k - 1]
        }
#pragma unroll
        for (int j = 0; j < D; ++j) vb[j * T * kWave] = y[j];                 // letter j, every lane
    };

    const int64_t ntiles = (L + T - 1) / T;
    for (int e = lane; e < T * D; e += kWave) gt[e] = 0.0f;
    fetch((ntiles - 1) * T);
    for (int64_t n = ntiles - 1; n >= 0; --n) {
        wave_lds_fence();
        stage();
        wave_lds_fence();
        fetch((n - 1) * T);                            // n = 0: out of range, zeros
#pragma unroll 1
        for (int tt = T - 1; tt >= 0; --tt) step(tt);
        wave_lds_fence();
        tile_reduce_uniform<D, T>(Vb, gt, D, lane, 0);     // the only writer of gt so far: plain read-modify-write
        wave_lds_fence();
        lane_chain_tile_reduce<D, KL, T, 0, KL>(Vb + D * T * kWave, gt, lane, letter);
        wave_lds_fence();
        if constexpr (POINTS) {
            // Point j of the row gets the gradient of segment j - 1 minus that of segment j.  The points at which the
            // segments of the tile walked before (pg, later in time) begin are complete now and are stored as one
            // aligned row; the first point of the row and the one after its last segment are left to the end.
            float* const row_points = grad_path + (b * P + seg0 + (n + 1) * T) * D;   // the same in every lane
            // (the lane number is taken through an opaque copy: addresses derived from it would otherwise be kept
            // in registers across the segment loop, which has none to spare)
            int lane_here = lane;
            asm volatile("" : "+v"(lane_here));
            for (int e = lane_here; e < T * D; e += kWave) {
                const int tt = e / D, i = e % D;
                if ((n + 1) * T + tt < L) row_points[e] = (tt >= 1 ? pg[e - D] : gt[(T - 1) * D + i]) - pg[e];
                if (n * T + tt == L - 1) cg[D + i] = gt[e];                  // last segment of the row
            }
            wave_lds_fence();
            for (int e = lane_here; e < T * D; e += kWave) {
                pg[e] = gt[e];
                gt[e] = 0.0f;
            }
            wave_lds_fence();
        } else {
            for (int e = lane; e < T * D; e += kWave) {
                const int64_t sgm = n * T + e / D;
                if (sgm < L) {
                    // windows of a path overlap: their gradients add up; rows that tile a path store
                    if (wl.win) unsafeAtomicAdd(gdx + (b * (P - 1) + seg0 + n * T) * D + e, gt[e]);
                    else gdx[(b * (P - 1) + seg0 + n * T) * D + e] = gt[e];
                }
                gt[e] = 0.0f;
            }
        }
    }
    if constexpr (POINTS) {
        // the points inside the first tile; then cg: gradient of the first segment of the row, cg + D: of its last one
        float* const row_points = grad_path + (b * P + seg0) * D;
        for (int e = lane; e < T * D; e += kWave) {
            const int tt = e / D;
            if (tt >= 1 && tt < L) row_points[e] = pg[e - D] - pg[e];
        }
        if (lane < D) cg[lane] = pg[lane];
        wave_lds_fence();
        if constexpr (CW == 0) {                       // the row is a whole path
            if (lane < D) {
                grad_path[(b * P) * D + lane] = -cg[lane];
                grad_path[(b * P + L) * D + lane] = cg[D + lane];
            }
        } else {
            float* const XY = smem + LY::OFF_XY;
            if (lane < 2 * D) XY[cib * 2 * D + lane] = cg[lane];
            __syncthreads();
            // point where chunk k begins (k = CW: the end of the path): last segment of chunk k - 1 minus first of k
            if ((int)threadIdx.x < (CW + 1) * D) {
                const int k = threadIdx.x / D, i = threadIdx.x % D;
                const float before = k >= 1 ? XY[(k - 1) * 2 * D + D + i] : 0.0f;
                const float after = k < CW ? XY[k * 2 * D + i] : 0.0f;
                const int64_t pt = k < CW ? k * Lc : P - 1;
                grad_path[(b * P + pt) * D + i] = before - after;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Backward on the vector ALU alone, for truncations whose words of length N - 2 fill whole wavefronts with room in
// the registers for two more levels: a lane holds a word u of length K = N - 2 (its chain of K letters per lane),
// the coefficients and adjoints of its D children and the gradients of the D^2 leaves below them.  The letters
// below u are the same in every lane, so the two lower levels are multiply-adds with lane-uniform increments and
// their gradient contributions are D per-letter sums (the matrix-core form of these levels, trunc_mfma_bwd_kernel,
// keeps the children in another lane layout and pays for the transposes: measured 20 % slower for d = 8).
// D^K / 64 wavefronts share a (path, chunk) row: the increment gradients are accumulated into gdx (zeroed by the
// caller) with floating-point atomics.
template <int D, int N, int T>
struct NodeLds {
    static constexpr int K = N - 2;
    static constexpr int NC = (N + 3) / 4 * 4;
    static constexpr int NSRC = D + K;                 // one source of gradient values per letter, one per chain letter
    // d = 8, depth 5: the sources of two segments stay in registers and are summed over lanes with cross-lane moves
    // (the LDS slots and their row sums cost a fifth of the kernel); other shapes park them in LDS (VB)
    static constexpr bool SOURCES_IN_REGISTERS = D == 8 && N == 5;
    static constexpr int OFF_GT = T * D * NC;
    // gradient tile [T][D]; with the sources in registers three of them (one per kind of source, stored, not
    // accumulated) and T values for the chain letter that is the same in the whole wavefront
    static constexpr int OFF_VB = OFF_GT + (SOURCES_IN_REGISTERS ? 3 * T * D + (T + 3) / 4 * 4 : T * D);
    static constexpr int PER_WAVE = OFF_VB + (SOURCES_IN_REGISTERS ? 0 : NSRC * T * kWave);
    static_assert(OFF_GT % 4 == 0 && OFF_VB % 4 == 0 && PER_WAVE % 4 == 0, "16-byte alignment of the LDS regions");
    static constexpr size_t BYTES = (size_t)kWavesPerBlock * PER_WAVE * sizeof(float);
};

// (the shortest tile is for launches with two wavefronts per SIMD: its registers are held to half a SIMD's)
template <int D, int N, int T>
__global__ __launch_bounds__(kWave * kWavesPerBlock, (D == 8 ? 2 : 1)) void trunc_node_bwd_kernel(
    const float* __restrict__ path, const float* __restrict__ coeffs, const float* __restrict__ grad,
    const float* __restrict__ coeffs_last, const float* __restrict__ grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc,
    WindowList wl, float* gdx, float* resid)
{
    static_assert((D & (D - 1)) == 0, "the gradient reduction takes letters as bit fields of the lane number");
    constexpr int K = N - 2;
    constexpr int WAVES = ipow(D, K) / kWave;          // wavefronts per row
    using LY = NodeLds<D, N, T>;
    static_assert(WAVES * kWave == ipow(D, K) && (LY::SOURCES_IN_REGISTERS || D * T <= kWave),
                  "whole wavefronts; one lane per (letter, segment) where the sources are summed from LDS");
    constexpr int NC = (N + 3) / 4 * 4;
    constexpr int EPL = (T * D + kWave - 1) / kWave;
    constexpr int LB = ilog2(D);
    extern __shared__ v4f bwd_smem[];

    const int lane = threadIdx.x % kWave;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // the same in every lane: scalar registers
    const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + wib;
    if (wave >= B * C * (wl.win ? wl.K : 1) * WAVES) return;
    float* const lds = (float*)bwd_smem + wib * LY::PER_WAVE;            // wave-private
    float (*Ec)[D][NC] = (float (*)[D][NC])lds;
    float* gt = lds + LY::OFF_GT;
    float* Vb = lds + LY::OFF_VB;
    const int64_t row = wave / WAVES;
    int64_t b, seg0, L;
    row_segments(wl, row, P, C, Lc, b, seg0, L);
    if (L <= 0) return;                                // an empty window: no gradient
    const int p = (int)(wave % WAVES) * kWave + lane;  // the lane's word of length K
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + (b * P + seg0) * D;
    const int64_t nW = level_start(D, N) + ipow(D, N);
    // rows of the last chunk of a path may live in arrays of their own ([B][|W|]); the others in a [B][C][|W|] array of
    // signatures and, then, a [B][C - 1][|W|] array of adjoints
    const bool in_last = coeffs_last != nullptr && row - b * C == C - 1;
    const float* cf = in_last ? coeffs_last + b * nW : coeffs + row * nW;
    const float* gr = in_last ? grad_last + b * nW : grad + (coeffs_last != nullptr ? row - b : row) * nW;

    // ---- state: signature and adjoints at the end of the row
    float Sc[K], Ac[K];                    // chain (a word shared by several lanes has its adjoint in the first of them)
    float S1[D], A1[D];                    // children of u
    float An[D][D];                        // gradients of the leaves: constant adjoints
    {
        int phi = 0;
#pragma unroll
        for (int k = 1; k <= K; ++k) {
            phi = phi * D + letter[k - 1];
            Sc[k - 1] = cf[level_start(D, k) + phi];
            Ac[k - 1] = p % ipow(D, K - k) == 0 ? gr[level_start(D, k) + phi] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < D; ++j) {
            S1[j] = cf[level_start(D, N - 1) + p * D + j];
            A1[j] = gr[level_start(D, N - 1) + p * D + j];
#pragma unroll
            for (int jj = 0; jj < D; ++jj) An[j][jj] = gr[level_start(D, N) + (p * D + j) * D + jj];
        }
    }

    float dxn[EPL];
    auto fetch = [&](int64_t j0) {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = (lane + q * kWave) < T * D ? lane + q * kWave : T * D - 1;
            int64_t jj = j0 + e / D;
            const bool ok = jj >= 0 && jj < L;
            jj = jj < 0 ? 0 : (jj < L ? jj : L - 1);
            const int i = e % D;
            const float x1 = X[(jj + 1) * D + i], x0 = X[jj * D + i];
            dxn[q] = ok ? x1 - x0 : 0.0f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = lane + q * kWave;
            if (e < T * D) {
#pragma unroll
                for (int t = 0; t < N; ++t) Ec[e / D][e % D][t] = dxn[q] * inv1(t);
            }
        }
    };

    // The scaled increments of a segment are read from LDS one segment ahead of their use (a lone wavefront per SIMD has
    // nobody to hide the LDS latency behind): `In` is what a step reads, filled by load_in while the step before runs.
    struct In {
        float ec[K][NC];                              // dX^{(letter[k])} / (t + 1) for the chain
        float eu[D][2];                               // dX^{(j)}, dX^{(j)} / 2: the same in every lane
    };
    auto load_in = [&](int row_t, In& in) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const float* src = &Ec[row_t][letter[k]][0];
#pragma unroll
            for (int t = 0; t <= N - (k + 1); ++t) in.ec[k][t] = src[t];
        }
#pragma unroll
        for (int j = 0; j < D; ++j) {
            in.eu[j][0] = Ec[row_t][j][0];
            in.eu[j][1] = Ec[row_t][j][1];
        }
    };
    // yo[D], co[K]: where the gradient sources of the segment go when they stay in registers
    auto step = [&](int row_t, const In& in, float* yo, float* co) {
        const float (&ec)[K][NC] = in.ec;
        const float (&eu)[D][2] = in.eu;
        // 1. reconstruction with -dX, 2. accumulators with +dX from the reconstructed signature
        float am[K + 1][N + 2], ap[K + 1][N + 2];
#pragma unroll
        for (int t = 0; t < N + 2; ++t) am[0][t] = ap[0][t] = 1.0f;
#pragma unroll
        for (int k = 1; k <= K; ++k) {
#pragma unroll
            for (int t = 1; t <= N - k; ++t) am[k][t] = fmaf(-ec[k - 1][t], am[k - 1][t + 1], Sc[k - 1]);
            Sc[k - 1] = fmaf(-ec[k - 1][0], am[k - 1][1], Sc[k - 1]);
#pragma unroll
            for (int t = 1; t <= N - k; ++t) ap[k][t] = fmaf(ec[k - 1][t], ap[k - 1][t + 1], Sc[k - 1]);
        }
        // 3. children and leaves: adjoint pushes and the gradient per letter
        float y[D];
#pragma unroll
        for (int j = 0; j < D; ++j) y[j] = 0.0f;
        const float hp2 = 0.5f * ap[K][2];
        float g1 = 0.0f, g2 = 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
            S1[j] = fmaf(-eu[j][0], am[K][1], S1[j]);
            const float Gp = fmaf(eu[j][1], ap[K][2], S1[j]);                 // A+[1] of the child
            float h = 0.0f;                                                    // its gbar[1], from the leaves
#pragma unroll
            for (int jj = 0; jj < D; ++jj) {
                h = fmaf(eu[jj][0], An[j][jj], h);
                y[jj] = fmaf(An[j][jj], Gp, y[jj]);                            // leaf letter jj
            }
            const float q0 = A1[j];
            A1[j] = q0 + h;
            y[j] = fmaf(q0, ap[K][1], y[j]);                                   // child letter j
            y[j] = fmaf(h, hp2, y[j]);
            g1 = fmaf(eu[j][0], q0, g1);                                       // what the child pushes up to u
            g2 = fmaf(eu[j][1], h, g2);
        }
        // 4. chain
        float gb[K + 1][N + 2];
#pragma unroll
        for (int k = 0; k <= K; ++k)
#pragma unroll
            for (int t = 0; t < N + 2; ++t) gb[k][t] = 0.0f;
        gb[K][1] = g1;
        gb[K][2] = g2;
        float* vb = Vb + row_t * kWave + lane;
#pragma unroll
        for (int k = K; k >= 1; --k) {
            gb[k][0] = Ac[k - 1];
            float gc = 0.0f, asum = 0.0f;
#pragma unroll
            for (int t = 0; t <= N - k; ++t) {
                const float q = gb[k][t];
                asum += q;
                gc = fmaf(q * inv1(t), ap[k - 1][t + 1], gc);
                gb[k - 1][t + 1] = fmaf(ec[k - 1][t], q, gb[k - 1][t + 1]);
            }
            Ac[k - 1] = asum;
            if constexpr (LY::SOURCES_IN_REGISTERS) co[k - 1] = gc;
            else vb[(D + k - 1) * T * kWave] = gc;                             // letter[k - 1]
        }
        if constexpr (LY::SOURCES_IN_REGISTERS) {
#pragma unroll
            for (int j = 0; j < D; ++j) yo[j] = y[j];
        } else {
#pragma unroll
            for (int j = 0; j < D; ++j) vb[j * T * kWave] = y[j];              // letter j, every lane
        }
    };
    // Sums over lanes for the two segments `first`, `first` + 1 (d = 8, depth 5: letter[2] = lane bits 0..2, letter[1] =
    // bits 3..5, letter[0] the same in the whole wavefront).  yv[8 s + j]: contribution of the lane to letter j in
    // segment s (every lane, every letter); cv[3 s + k]: contribution to letter[k].  Exchange rounds that halve the
    // number of values come first (across the halves and rows of the wavefront: swap instructions), plain butterfly
    // sums last; the partners used (lane ^ 32, ^ 16, ^ 8, ^ 7, ^ 3, ^ 1) generate every lane.  Results are stored, one
    // tile per kind of source: every (segment, letter) entry of a tile has exactly one writer per tile.
    float* const gy = gt;
    float* const g1 = gt + T * D;
    float* const g2 = gt + 2 * T * D;
    float* const gc0 = gt + 3 * T * D;
    auto reduce_pair = [&](int first, const float* yv, const float* cv) {
        auto r8 = [](float x) { return dpp_lane<0x128>(x); };      // lane ^ 8
        auto m7 = [](float x) { return dpp_lane<0x141>(x); };      // lane ^ 7
        auto q3 = [](float x) { return dpp_lane<0x1B>(x); };       // lane ^ 3
        auto q1 = [](float x) { return dpp_lane<0xB1>(x); };       // lane ^ 1
        // letters below the lane's word: lane bit 5 ends with the segment, bits 4, 3, 2 with the letter
        float a[D / 2];
#pragma unroll
        for (int i = 0; i < D / 2; ++i)
            a[i] = fold_swap16(fold_swap32(yv[i], yv[D + i]), fold_swap32(yv[i + D / 2], yv[D + i + D / 2]));
        fold_halves<4>(a, (lane & 8) != 0, r8);
        fold_halves<2>(a, (lane & 4) != 0, m7);
        float ry = a[0];
        ry += q3(ry);
        ry += q1(ry);
        if ((lane & 3) == 0) gy[(first + (lane >> 5)) * D + ((lane >> 2) & 7)] = ry;
        // letter[0]: all 64 lanes
        float r0 = fold_swap32(cv[0], cv[K]);
        r0 = fold_swap16(r0, r0);
        r0 += r8(r0);
        r0 += m7(r0);
        r0 += q3(r0);
        r0 += q1(r0);
        if ((lane & 31) == 0) gc0[first + (lane >> 5)] = r0;
        // letter[1]: the eight lanes that differ in bits 0..2
        float c1[2] = {cv[1], cv[K + 1]};
        fold_halves<2>(c1, (lane & 4) != 0, m7);
        float r1 = c1[0];
        r1 += q3(r1);
        r1 += q1(r1);
        if ((lane & 3) == 0) g1[(first + ((lane >> 2) & 1)) * D + letter[1]] = r1;
        // letter[2]: the eight lanes that differ in bits 3..5
        float r2 = fold_swap32(cv[2], cv[K + 2]);
        r2 = fold_swap16(r2, r2);
        r2 += r8(r2);
        if ((lane & 0x18) == 0) g2[(first + (lane >> 5)) * D + letter[2]] = r2;
    };

    const int64_t ntiles = (L + T - 1) / T;
    for (int e = lane; e < T * D; e += kWave) gt[e] = 0.0f;
    fetch((ntiles - 1) * T);
    for (int64_t n = ntiles - 1; n >= 0; --n) {
        wave_lds_fence();
        stage();
        wave_lds_fence();
        fetch((n - 1) * T);                            // n = 0: out of range, zeros
        if constexpr (LY::SOURCES_IN_REGISTERS) {
            static_assert(K == 3 && T % 2 == 0 && T >= 4, "reduce_pair is written for three chain letters");
            In ia, ib;
            float yv[2 * D], cv[2 * K];
            load_in(T - 1, ia);
#pragma unroll 1
            for (int tt = T - 1; tt >= 3; tt -= 2) {
                load_in(tt - 1, ib);
                step(tt, ia, yv + D, cv + K);
                load_in(tt - 2, ia);
                step(tt - 1, ib, yv, cv);
                reduce_pair(tt - 1, yv, cv);
            }
            load_in(0, ib);
            step(1, ia, yv + D, cv + K);
            step(0, ib, yv, cv);
            reduce_pair(0, yv, cv);
            wave_lds_fence();
        } else {
            static_assert(T % 2 == 0 && T >= 4, "the segment loop is unrolled by two");
            In ia, ib;
            load_in(T - 1, ia);
#pragma unroll 1
            for (int tt = T - 1; tt >= 3; tt -= 2) {
                load_in(tt - 1, ib);
                step(tt, ia, nullptr, nullptr);
                load_in(tt - 2, ia);
                step(tt - 1, ib, nullptr, nullptr);
            }
            load_in(0, ib);
            step(1, ia, nullptr, nullptr);
            step(0, ib, nullptr, nullptr);
            wave_lds_fence();
            tile_reduce_uniform<D, T>(Vb, gt, D, lane, 0);     // the only writer of gt so far: plain read-modify-write
            wave_lds_fence();
            tile_reduce<(1 << LB) - 1, T>(Vb + (D + K - 1) * T * kWave, gt, D, lane, letter[K - 1]);
            chain_tile_reduce<D, K, T, 0>(Vb + D * T * kWave, gt, lane, letter);
            wave_lds_fence();
        }
        // flush: (segment, letter) is contiguous in gdx
        for (int e = lane; e < T * D; e += kWave) {
            const int64_t sg = n * T + e / D;
            float v;
            if constexpr (LY::SOURCES_IN_REGISTERS) {
                v = (gy[e] + g1[e]) + (g2[e] + (e % D == letter[0] ? gc0[e / D] : 0.0f));
            } else {
                v = gt[e];
                gt[e] = 0.0f;
            }
            if (sg < L) unsafeAtomicAdd(gdx + (b * (P - 1) + seg0 + n * T) * D + e, v);
        }
    }
    if (resid != nullptr && seg0 == 0) {
        float m = 0.0f;
#pragma unroll
        for (int k = 0; k < K; ++k) m = fmaxf(m, fabsf(Sc[k]));
#pragma unroll
        for (int j = 0; j < D; ++j) m = fmaxf(m, fabsf(S1[j]));
        report_residual(m, resid, b);
    }
}

template <int D, int N, int T = 8>
hipError_t launch_trunc_node_bwd(const float* path, const float* coeffs, const float* grad, const float* coeffs_last,
                                 const float* grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc, float* gdx, float* resid,
                                 hipStream_t stream, const WindowList& wl = WindowList())
{
    using LY = NodeLds<D, N, T>;
    static_assert(LY::BYTES <= 160 * 1024, "LDS of one compute unit");
    const int64_t waves = B * C * (wl.win ? wl.K : 1) * (ipow(D, N - 2) / kWave);
    const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (LY::BYTES > 64 * 1024) {                 // above the default limit the kernel has to be told once
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&trunc_node_bwd_kernel<D, N, T>), (int)LY::BYTES);
        if (e != hipSuccess) return e;
    }
    trunc_node_bwd_kernel<D, N, T><<<(unsigned)blocks, kWave * kWavesPerBlock, LY::BYTES, stream>>>(
        path, coeffs, grad, coeffs_last, grad_last, B, P, C, Lc, wl, gdx, resid);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// Forward in the same register layout, for batches too short to fill the chip with one wavefront per path: a
// workgroup is one path, cut into CW time chunks; a chunk is shared by D / TW wavefronts that hold TW of the D tails
// (and everything below them) each and all recompute the chain above the tails.  Every wavefront runs the
// recursion over its chunk from the identity and publishes its part of the chunk signature to LDS; the workgroup
// then multiplies the chunk signatures (Chen's relation; CW = 4: (S_1 S_2)(S_3 S_4)) and writes the last product
// to coeffs.  Nothing but the path is read and nothing but the signature is written.  (Two chunks stay the faster
// form for large batches too: measured against a single chunk per path up to 8,192 paths.)
template <int D, int N, int T, int CW, int TW>
struct TailsFwdLds {
    static constexpr int NC = (N + 3) / 4 * 4;
    static constexpr int H = D / TW;
    static constexpr int NWV = CW * H;
    static constexpr int W = level_start(D, N) + ipow(D, N);
    static constexpr int TILE = T * 2 * D + T * D * NC;                      // E, Ec of one wavefront
    static constexpr int NBUF = CW == 2 ? 2 : CW + 2;                        // chunk signatures and first-round products
    static constexpr int OFF_S = NWV * TILE;
    static constexpr int TOTAL = OFF_S + NBUF * W;
    static_assert(CW == 2 || CW == 4, "two or four chunks per workgroup");
    static_assert(TILE % 4 == 0 && W % 4 == 0, "16-byte alignment");
    static constexpr size_t BYTES = (size_t)TOTAL * sizeof(float);
};

template <int D, int N, int T, int CW, int TW>
__global__ __launch_bounds__(kWave * CW * (D / TW)) void trunc_tails_fwd_kernel(const float* __restrict__ path, int64_t P,
                                                                               int64_t Lc, WindowList wl,
                                                                               float* __restrict__ coeffs)
{
    static_assert(D == 4, "one group of four letters");
    constexpr int K = N - 2;                          // length of the tail words
    constexpr int KL = K - 1;                         // letters held per lane
    static_assert(ipow(D, KL) == kWave, "64 words of length N - 3, one per lane");
    constexpr int NC = (N + 3) / 4 * 4;
    constexpr int EPL = (T * D + kWave - 1) / kWave;
    using LY = TailsFwdLds<D, N, T, CW, TW>;
    constexpr int H = LY::H;
    constexpr int W = LY::W;
    extern __shared__ v4f fwd_smem[];

    const int lane = threadIdx.x % kWave;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // the same in every lane: scalar registers
    const int cib = wib / H;                          // chunk of the workgroup's path
    const int i0 = (wib % H) * TW;                    // first tail of this wavefront
    const bool first = wib % H == 0;
    // the workgroup's row: a path, or with a window list a (path, window) pair whose segments are cut into CW chunks
    // (an empty window or chunk leaves the identity, which the products carry along)
    const int64_t orow = blockIdx.x;
    int64_t b = orow, seg0 = cib * Lc, L = (P - 1 - seg0) < Lc ? (P - 1 - seg0) : Lc;
    if (wl.win != nullptr) {
        int64_t l0, lrow;
        row_segments(wl, orow, P, 1, 0, b, l0, lrow);
        const int64_t lc = (lrow + CW - 1) / CW;
        seg0 = l0 + cib * lc;
        L = lrow - cib * lc < lc ? lrow - cib * lc : lc;
        L = L < 0 ? 0 : L;
    }
    float* const smem = (float*)fwd_smem;
    float (*E)[2][D] = (float (*)[2][D])(smem + wib * LY::TILE);            // wave-private
    float (*Ec)[D][NC] = (float (*)[D][NC])(smem + wib * LY::TILE + T * 2 * D);
    float* const SB = smem + LY::OFF_S;
    int letter[KL];
    {
        int q = lane;
#pragma unroll
        for (int k = KL - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + (b * P + seg0) * D;

    float Sc[KL];                          // per-lane chain
    float St[TW];                          // tails i0 .. i0 + TW - 1
    v4f S1[TW];                            // slice level: children of the tails (child layout)
    v4f S2[TW][4];                         // leaves (child layout)
#pragma unroll
    for (int k = 0; k < KL; ++k) Sc[k] = 0.0f;
    const v4f zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int ii = 0; ii < TW; ++ii) {
        St[ii] = 0.0f;
        S1[ii] = zero4;
#pragma unroll
        for (int r = 0; r < 4; ++r) S2[ii][r] = zero4;
    }

    float dxn[EPL];
    auto fetch = [&](int64_t j0) {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = (lane + q * kWave) < T * D ? lane + q * kWave : T * D - 1;
            int64_t jj = j0 + e / D;
            const bool ok = jj < L;
            jj = jj < L ? jj : (L > 0 ? L - 1 : 0);
            const int i = e % D;
            const float x1 = X[(jj + (L > 0 ? 1 : 0)) * D + i], x0 = X[jj * D + i];   // an empty chunk reads its own point
            dxn[q] = ok ? x1 - x0 : 0.0f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const int e = lane + q * kWave;
            if (e < T * D) {
#pragma unroll
                for (int t = 0; t < N; ++t) {
                    const float v = dxn[q] * inv1(t);
                    if (t < 2) E[e / D][t][e % D] = v;
                    Ec[e / D][e % D][t] = v;
                }
            }
        }
    };
    // matrix-core B operand: lanes 0..15 carry dX^{(lane % 4)}, lanes 16..31 dX^{(lane % 4)} / 2
    const int offB = lane < 32 ? (lane / 16) * D + (lane & 3) : 0;

    const int64_t nt = (L + T - 1) / T;
    fetch(0);
    for (int64_t n = 0; n < nt; ++n) {
        wave_lds_fence();
        stage();
        wave_lds_fence();
        fetch((n + 1) * T);                            // beyond the chunk: zeros
#pragma unroll 2
        for (int tt = 0; tt < T; ++tt) {
            const float bs = E[tt][0][offB];
            float a[KL + 1][N + 2];
#pragma unroll
            for (int t = 0; t < N + 2; ++t) a[0][t] = 1.0f;
#pragma unroll
            for (int k = 1; k <= KL; ++k) {
                const float* src = &Ec[tt][letter[k - 1]][0];
#pragma unroll
                for (int t = 1; t <= N - k; ++t) a[k][t] = fmaf(src[t], a[k - 1][t + 1], Sc[k - 1]);
                Sc[k - 1] = fmaf(src[0], a[k - 1][1], Sc[k - 1]);
            }
#pragma unroll
            for (int ii = 0; ii < TW; ++ii) {
                const float* et = &Ec[tt][i0 + ii][0];
                const float a1 = fmaf(et[1], a[KL][2], St[ii]);
                const float a2 = fmaf(et[2], a[KL][3], St[ii]);
                St[ii] = fmaf(et[0], a[KL][1], St[ii]);
                const v4f Gq = mfma4(a2, bs, S1[ii], 1);
                S1[ii] = mfma4(a1, bs, S1[ii], 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) S2[ii][r] = mfma4(Gq[r], bs, S2[ii][r], 0);
            }
        }
    }
    {   // publish the chunk signature in canonical order
        float* out = SB + cib * W;
        int phi = 0;
#pragma unroll
        for (int k = 1; k <= KL; ++k) {
            phi = phi * D + letter[k - 1];
            if (first && lane % ipow(D, KL - k) == 0) out[level_start(D, k) + phi] = Sc[k - 1];
        }
#pragma unroll
        for (int ii = 0; ii < TW; ++ii) {
            const int i = i0 + ii;
            out[level_start(D, K) + lane * D + i] = St[ii];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // register r: child (letter lane % 4) of tail i of lane 4 blk + r; (r, rr): child (letter lane % 4) of
                // the slice word (r, lane 4 blk + rr)
                out[level_start(D, N - 1) + (((lane & ~3) + r) * D + i) * D + (lane & 3)] = S1[ii][r];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    out[level_start(D, N) + ((((lane & ~3) + r) * D + i) * D + rr) * D + (lane & 3)] = S2[ii][r][rr];
            }
        }
    }
    __syncthreads();
    constexpr int NT = LY::NWV * kWave;
    float* const dst = coeffs + orow * W;
    if constexpr (CW == 4) {
        float* const TB = SB + CW * W;
        lds_tensor_product<D, N>(SB, SB + W, TB, threadIdx.x, NT);
        lds_tensor_product<D, N>(SB + 2 * W, SB + 3 * W, TB + W, threadIdx.x, NT);
        __syncthreads();
        lds_tensor_product<D, N>(TB, TB + W, dst, threadIdx.x, NT);
    } else {
        lds_tensor_product<D, N>(SB, SB + W, dst, threadIdx.x, NT);
    }
}

template <int D, int N, int CW, int TW>
hipError_t launch_trunc_tails_fwd(const float* path, int64_t B, int64_t P, int64_t Lc, float* coeffs, hipStream_t stream,
                                  const WindowList& wl = WindowList())
{
    constexpr int T = 8;
    using LY = TailsFwdLds<D, N, T, CW, TW>;
    static_assert(LY::BYTES <= 160 * 1024, "LDS of one compute unit");
    const int64_t rows = B * (wl.win ? wl.K : 1);
    if ((!wl.win && (CW - 1) * Lc >= P - 1) || rows > 0x7fffffff) return hipErrorInvalidValue;   // every chunk holds a segment
    if (LY::BYTES > 64 * 1024) {                 // above the default limit the kernel has to be told once
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&trunc_tails_fwd_kernel<D, N, T, CW, TW>), (int)LY::BYTES);
        if (e != hipSuccess) return e;
    }
    trunc_tails_fwd_kernel<D, N, T, CW, TW><<<(unsigned)rows, kWave * LY::NWV, LY::BYTES, stream>>>(path, P, Lc, wl, coeffs);
    return hipGetLastError();
}

template <int D, int N, int CW, bool POINTS>
hipError_t launch_trunc_tails_bwd(const float* path, const float* coeffs, const float* grad, int64_t B, int64_t P,
                                  int64_t C, int64_t Lc, float* out, hipStream_t stream, const WindowList& wl = WindowList())
{
    constexpr int T = 8;
    using LY = TailsLds<D, N, T, CW>;
    static_assert(LY::BYTES <= 160 * 1024, "LDS of one compute unit");
    if (CW && C != CW) return hipErrorInvalidValue;
    if (wl.win && (CW != 0 || POINTS || C != 1)) return hipErrorInvalidValue;   // windows: one row each, gradients added up
    const int64_t blocks = CW ? B : (B * C * (wl.win ? wl.K : 1) + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (LY::BYTES > 64 * 1024) {                 // above the default limit the kernel has to be told once
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&trunc_tails_bwd_kernel<D, N, T, CW, POINTS>), (int)LY::BYTES);
        if (e != hipSuccess) return e;
    }
    if (POINTS && CW == 0 && C != 1) return hipErrorInvalidValue;   // rows that are parts of paths cannot apply the chain rule
    trunc_tails_bwd_kernel<D, N, T, CW, POINTS><<<(unsigned)blocks, kWave * LY::NWV, LY::BYTES, stream>>>(path, coeffs, grad, B, P,
                                                                                                        C, Lc, wl, out);
    return hipGetLastError();
}

template <int D, int N, int WQ, int T, int VG = T>
hipError_t launch_trunc_mfma_bwd(const float* path, const float* coeffs, const float* grad, const float* coeffs_last,
                                 const float* grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc, float* gdx, float* resid,
                                 hipStream_t stream, const WindowList& wl = WindowList())
{
    using G = MGeo<D, N, N - 2, WQ>;
    using LY = BwdLds<D, N, WQ, T, VG>;
    static_assert(LY::BYTES <= 160 * 1024, "LDS of one compute unit");
    const int64_t waves = B * C * (wl.win ? wl.K : 1) * G::WAVES;
    const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (LY::BYTES > 64 * 1024) {                 // above the default limit the kernel has to be told once
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&trunc_mfma_bwd_kernel<D, N, WQ, T, VG>), (int)LY::BYTES);
        if (e != hipSuccess) return e;
    }
    trunc_mfma_bwd_kernel<D, N, WQ, T, VG><<<(unsigned)blocks, kWave * kWavesPerBlock, LY::BYTES, stream>>>(
        path, coeffs, grad, coeffs_last, grad_last, B, P, C, Lc, wl, gdx, resid);
    return hipGetLastError();
}

}  // namespace

// (D, N) pairs with a register-resident kernel, and the unit shape used for each.
bool trunc_forward_available(int d, int depth)
{
    return (d == 4 && depth == 6) || (d == 8 && depth == 5) || (d == 16 && depth == 4);
}

// d = 4, depth 6 forward: chain of four letters on the vector ALU, two cascade levels on the matrix cores, four
// wavefronts per path.  (A chain of three letters - one wavefront per path, three cascade levels, 168 registers -
// also works with this kernel; with time chunks it was no faster on 256 paths of 256 segments.)
constexpr int kChainFwd46 = 4;
constexpr int kOccFwd46 = 4;

// Workgroups of the kernels that fit on one compute unit at a time (= wavefronts per SIMD), from the registers
// and LDS each instantiation uses; the launcher of time chunks sizes the number of chunks with it.
int trunc_occupancy(int d, int depth, int backward)
{
    if (d == 4 && depth == 6) return backward ? 3 : kOccFwd46;
    if (d == 8 && depth == 5) return backward ? 1 : 2;     // forward: 216 and 204 registers under the scheduler that
    if (d == 16 && depth == 4) return backward ? 1 : 2;    // maximises instruction-level parallelism
    return 1;
}

// wavefronts one (path, chunk) row occupies
int trunc_waves_per_row(int d, int depth, int backward)
{
    if (d == 4 && depth == 6) return backward ? MGeo<4, 6, 4, 1>::WAVES : MGeo<4, 6, kChainFwd46, 1>::WAVES;
    if (d == 8 && depth == 5) return backward ? MGeo<8, 5, 3, 2>::WAVES : MGeo<8, 5, 3, 2>::WAVES;
    if (d == 16 && depth == 4) return backward ? MGeo<16, 4, 2, 1>::WAVES : MGeo<16, 4, 2, 1>::WAVES;
    return 1;
}

// C chunks of Lc segments per path (C = 1, Lc = P - 1: whole paths); coeffs has B * C rows
hipError_t trunc_forward(int d, int depth, const float* path, int64_t B, int64_t P, int64_t C, int64_t Lc, float* coeffs,
                         hipStream_t stream)
{
    if (B * C > 65535 * 16) return hipErrorInvalidValue;
    if (d == 4 && depth == 6) return launch_trunc_mfma_fwd<4, 6, kChainFwd46, 1>(path, B, P, C, Lc, coeffs, stream);
    if (d == 8 && depth == 5) return launch_trunc_mfma_fwd<8, 5, 3, 2>(path, B, P, C, Lc, coeffs, stream);
    if (d == 16 && depth == 4) return launch_trunc_mfma_fwd<16, 4, 2, 1>(path, B, P, C, Lc, coeffs, stream);
    return hipErrorInvalidValue;
}

bool trunc_backward_available(int d, int depth)
{
    return (d == 4 && depth == 6) || (d == 8 && depth == 5) || (d == 16 && depth == 4);
}

// One wavefront per (path, chunk) row; every segment of every path must be covered by exactly one row (the kernel
// stores, it does not accumulate).
bool trunc_backward_tails_available(int d, int depth) { return d == 4 && depth == 6; }

// grad_path given (C = 1 only): the chain rule is applied in the kernel and gdx is not used
hipError_t trunc_backward_tails(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                                int64_t P, int64_t C, int64_t Lc, float* gdx, float* grad_path, hipStream_t stream)
{
    if (!(d == 4 && depth == 6)) return hipErrorInvalidValue;
    if (grad_path) return launch_trunc_tails_bwd<4, 6, 0, true>(path, coeffs, grad_coeffs, B, P, C, Lc, grad_path, stream);
    return launch_trunc_tails_bwd<4, 6, 0, false>(path, coeffs, grad_coeffs, B, P, C, Lc, gdx, stream);
}

// Fused form: the C (2, 4 or 8) chunks of a path are the wavefronts of one workgroup; coeffs / grad_coeffs are the
// terminal signature and its gradient [B, |W|], nothing else is needed, and the gradient with respect to the points
// [B, P, d] is written directly.  Every chunk must hold at least one segment.
hipError_t trunc_backward_tails_fused(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs,
                                      int64_t B, int64_t P, int64_t C, int64_t Lc, float* grad_path, hipStream_t stream)
{
    if ((C - 1) * Lc >= P - 1 || !grad_path) return hipErrorInvalidValue;
    if (!(d == 4 && depth == 6)) return hipErrorInvalidValue;
    if (C == 8) return launch_trunc_tails_bwd<4, 6, 8, true>(path, coeffs, grad_coeffs, B, P, C, Lc, grad_path, stream);
    if (C == 4) return launch_trunc_tails_bwd<4, 6, 4, true>(path, coeffs, grad_coeffs, B, P, C, Lc, grad_path, stream);
    if (C == 2) return launch_trunc_tails_bwd<4, 6, 2, true>(path, coeffs, grad_coeffs, B, P, C, Lc, grad_path, stream);
    return hipErrorInvalidValue;
}

// Forward with the C = 2 or 4 chunks of a path in one workgroup (d = 4, depth 6); coeffs 16-byte aligned
bool trunc_forward_tails_available(int d, int depth) { return d == 4 && depth == 6; }

hipError_t trunc_forward_tails_fused(int d, int depth, const float* path, int64_t B, int64_t P, int64_t C, int64_t Lc,
                                     float* coeffs, hipStream_t stream)
{
    if (!(d == 4 && depth == 6)) return hipErrorInvalidValue;
    if (C == 4) return launch_trunc_tails_fwd<4, 6, 4, 2>(path, B, P, Lc, coeffs, stream);
    if (C == 2) return launch_trunc_tails_fwd<4, 6, 2, 2>(path, B, P, Lc, coeffs, stream);
    return hipErrorInvalidValue;
}

const char* trunc_backward_kernel_name(int d, int depth)
{
    return (d == 16 && depth == 4) ? "trunc_mfma_bwd_kernel" : "trunc_node_bwd_kernel";
}

// gdx: [B, L, d] accumulation buffer, zeroed by the caller
hipError_t trunc_backward(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs,
                          const float* coeffs_last, const float* grad_last, int64_t B, int64_t P, int64_t C, int64_t Lc,
                          float* gdx, float* resid, int tile, hipStream_t stream)
{
    if ((coeffs_last == nullptr) != (grad_last == nullptr)) return hipErrorInvalidValue;
    if (d == 4 && depth == 6)
        return launch_trunc_node_bwd<4, 6>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
    // d = 8: with the gradient sources in registers a wavefront needs a few KB of LDS whatever the tile; the tile length
    // only sets how often increments are staged and gradients flushed
    if (d == 8 && depth == 5) {
        if (tile == 4) return launch_trunc_node_bwd<8, 5, 4>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
        if (tile == 16) return launch_trunc_node_bwd<8, 5, 16>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
        return launch_trunc_node_bwd<8, 5, 8>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
    }
    // d = 16: a tile of 16 segments fills the 16 columns of the time-batched matrix products.  With the gradient sources
    // parked in LDS for the whole tile a workgroup takes 126 KB, one per compute unit, and a lone wavefront issues vector
    // instructions at half the rate of its SIMD: that form (segments software-pipelined) is for launches that have no
    // second wavefront per SIMD to offer anyway.  With the sources of 4 segments in registers, summed by cross-lane moves,
    // the workgroup needs 78 KB and two share a compute unit: taken from 2,048 wavefronts on.  tile = 16 / 4 force the
    // two forms; 12 and 8 are shorter tiles (three quarters, half of the columns), measured slower, kept selectable.
    if (d == 16 && depth == 4) {
        const int t = tile == 4 || tile == 8 || tile == 12 || tile == 16 ? tile : (B * C * 16 >= 2048 ? 4 : 16);
        if (t == 4) return launch_trunc_mfma_bwd<16, 4, 1, 16, 4>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
        if (t == 8) return launch_trunc_mfma_bwd<16, 4, 1, 8>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
        if (t == 12) return launch_trunc_mfma_bwd<16, 4, 1, 12, 4>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
        return launch_trunc_mfma_bwd<16, 4, 1, 16>(path, coeffs, grad_coeffs, coeffs_last, grad_last, B, P, C, Lc, gdx, resid, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t trunc_forward_windows(int d, int depth, const float* path, int64_t B, int64_t P, const WindowList& wl, float* coeffs,
                                 hipStream_t stream)
{
    if (!wl.win || wl.K < 1 || B * wl.K > 65535) return hipErrorInvalidValue;
    // d = 4: the two halves of a window in one workgroup (16-byte aligned rows), as for whole paths
    if (d == 4 && depth == 6) {
        if (((uintptr_t)coeffs & 15) == 0) return launch_trunc_tails_fwd<4, 6, 2, 2>(path, B, P, 0, coeffs, stream, wl);
        return launch_trunc_mfma_fwd<4, 6, kChainFwd46, 1>(path, B, P, 1, P - 1, coeffs, stream, wl);
    }
    if (d == 8 && depth == 5) return launch_trunc_mfma_fwd<8, 5, 3, 2>(path, B, P, 1, P - 1, coeffs, stream, wl);
    if (d == 16 && depth == 4) return launch_trunc_mfma_fwd<16, 4, 2, 1>(path, B, P, 1, P - 1, coeffs, stream, wl);
    return hipErrorInvalidValue;
}

hipError_t trunc_backward_windows(int d, int depth, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                                  int64_t P, const WindowList& wl, float* gdx, hipStream_t stream)
{
    if (!wl.win || wl.K < 1 || B * wl.K > 65535) return hipErrorInvalidValue;
    if (d == 4 && depth == 6)
        return launch_trunc_tails_bwd<4, 6, 0, false>(path, coeffs, grad_coeffs, B, P, 1, P - 1, gdx, stream, wl);
    if (d == 8 && depth == 5) {
        const bool small = B * wl.K * 8 >= 2048;           // see trunc_backward
        return small ? launch_trunc_node_bwd<8, 5, 4>(path, coeffs, grad_coeffs, nullptr, nullptr, B, P, 1, P - 1, gdx, nullptr, stream, wl)
                     : launch_trunc_node_bwd<8, 5, 8>(path, coeffs, grad_coeffs, nullptr, nullptr, B, P, 1, P - 1, gdx, nullptr, stream, wl);
    }
    if (d == 16 && depth == 4)
        return launch_trunc_mfma_bwd<16, 4, 1, 16>(path, coeffs, grad_coeffs, nullptr, nullptr, B, P, 1, P - 1, gdx, nullptr, stream, wl);
    return hipErrorInvalidValue;
}

}  // namespace sig
