// Full truncations of any alphabet size with lanes = words: kernels compiled at run time (hiprtc) from one fixed
// source with the shape (d, N) as macros, because the register arrays below are sized by d.
//
// Layout (the one of trunc_node_bwd_kernel, without its power-of-two assumptions): a lane holds a word u of length
// K = N - R together with everything below it, R = 1 (the d leaves under u) or R = 2 (d children and d^2 leaves).
// The coefficients of u's prefixes (the chain) are recomputed in every lane that shares them and stored by one.
// The letters below u are the same in every lane, so those levels are multiply-adds with lane-uniform increments
// (Section 3.1, eq. (3) and Algorithm 1, with the Horner intermediates shared between words).  ceil(d^K / 64)
// wavefronts serve a path; lanes past d^K carry a copy of the last word with zero adjoints and store nothing.
// Against lanes = paths this fills the wavefronts for any batch size and needs one short compilation per shape
// instead of one that grows with the word set.
#include <sstream>
#include <string>

#include "jit.hpp"

namespace sig {
namespace {

const char* const kLanesSource = R"SRC(
#define K (N - R)
#define NC ((N + 3) / 4 * 4)
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int ipow(int b, int e)
{
    int r = 1;
    for (int q = 0; q < e; ++q) r *= b;
    return r;
}
// first canonical index of the words of length n >= 1
constexpr long level_start(int n)
{
    long r = 0;
    for (int m = 1; m < n; ++m) r += ipow(D, m);
    return r;
}
constexpr float inv1(int t) { return 1.0f / (float)(t + 1); }

#define NL ipow(D, K)                       /* words of length K = lanes per path */
#define WAVES ((NL + 63) / 64)
#define NWORDS (level_start(N) + ipow(D, N))

static_assert(K >= 1 && (R == 1 || R == 2), "a lane holds a word of length N - R and one or two levels below it");
static_assert(T * D <= 64, "one lane per (letter, segment) of a tile");

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// increment (segment j0 + lane / D, letter lane % D) of the tile that starts at segment j0; zero outside [0, L)
__device__ __forceinline__ float fetch_increment(const float* __restrict__ X, long j0, long L, int lane)
{
    const int e = lane < T * D ? lane : T * D - 1;
    long jj = j0 + e / D;
    const bool ok = jj >= 0 && jj < L;
    jj = jj < 0 ? 0 : (jj < L ? jj : L - 1);
    const int i = e % D;
    const float x1 = X[(jj + 1) * D + i], x0 = X[jj * D + i];
    return ok ? x1 - x0 : 0.0f;
}
// Ec[segment][letter][t] = dX / (t + 1)
__device__ __forceinline__ void stage_increment(float* Ec, float dx, int lane)
{
    if (lane < T * D) {
#pragma unroll
        for (int t = 0; t < N; ++t) Ec[lane * NC + t] = dx * inv1(t);
    }
}

#if !BACKWARD
extern "C" __global__ __launch_bounds__(64 * NWB) void sig_fwd_lanes(const float* __restrict__ path, long B, long P,
                                                                      float* __restrict__ coeffs)
{
    __shared__ __attribute__((aligned(16))) float smem[NWB * T * D * NC];
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long wave = (long)blockIdx.x * NWB + wib;
    if (wave >= B * WAVES) return;                       // wavefronts share nothing: no barrier is skipped
    float* Ec = smem + wib * (T * D * NC);
    const long b = wave / WAVES;
    const int p0 = __builtin_amdgcn_readfirstlane((int)(wave - b * WAVES) * 64);
    const bool valid = p0 + lane < NL;
    const int p = valid ? p0 + lane : NL - 1;
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + b * P * D;
    const long L = P - 1;

    float Sc[K], S1[D];
#pragma unroll
    for (int k = 0; k < K; ++k) Sc[k] = 0.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) S1[j] = 0.0f;
#if R == 2
    float S2[D][D];
#pragma unroll
    for (int j = 0; j < D; ++j)
#pragma unroll
        for (int jj = 0; jj < D; ++jj) S2[j][jj] = 0.0f;
#endif

    const long ntiles = (L + T - 1) / T;
    float dxn = fetch_increment(X, 0, L, lane);
    for (long n = 0; n < ntiles; ++n) {
        wave_lds_fence();
        stage_increment(Ec, dxn, lane);
        wave_lds_fence();
        dxn = fetch_increment(X, (n + 1) * T, L, lane);  // past the end: zeros, and a zero increment changes nothing
#pragma unroll 2
        for (int tt = 0; tt < T; ++tt) {
            const float* Et = Ec + tt * D * NC;
            float ap[K + 1][N + 2];
#pragma unroll
            for (int t = 0; t < N + 2; ++t) ap[0][t] = 1.0f;
#pragma unroll
            for (int k = 1; k <= K; ++k) {
                const float* src = Et + letter[k - 1] * NC;
#pragma unroll
                for (int t = 1; t <= N - k; ++t) ap[k][t] = __builtin_fmaf(src[t], ap[k - 1][t + 1], Sc[k - 1]);
                Sc[k - 1] = __builtin_fmaf(src[0], ap[k - 1][1], Sc[k - 1]);
            }
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const float e0 = Et[j * NC];
#if R == 2
                const float Gp = __builtin_fmaf(Et[j * NC + 1], ap[K][2], S1[j]);
#pragma unroll
                for (int jj = 0; jj < D; ++jj) S2[j][jj] = __builtin_fmaf(Et[jj * NC], Gp, S2[j][jj]);
#endif
                S1[j] = __builtin_fmaf(e0, ap[K][1], S1[j]);
            }
        }
    }

    if (!valid) return;
    float* out = coeffs + b * NWORDS;
#pragma unroll
    for (int k = 1; k <= K; ++k)
        if (p % ipow(D, K - k) == 0) out[level_start(k) + p / ipow(D, K - k)] = Sc[k - 1];
#pragma unroll
    for (int j = 0; j < D; ++j) {
        out[level_start(K + 1) + (long)p * D + j] = S1[j];
#if R == 2
#pragma unroll
        for (int jj = 0; jj < D; ++jj) out[level_start(K + 2) + ((long)p * D + j) * D + jj] = S2[j][jj];
#endif
    }
}

#else
// Backward (Section 4: reconstruction with -dX, Proposition 4.6; gradient of Proposition 4.1 in its adjoint form).
// Per segment a lane produces one gradient contribution per letter below u (all lanes to the same letter) and one
// per chain letter (to the lane's own letter at that position); they go to LDS per segment of a tile and lane
// j T + t then sums, for letter j and segment t, the rows of the first kind and the members of the second kind,
// and adds the total to gdx (zeroed by the caller) with one floating-point atomic.
#define NSRC (D + K)
#define BW_PER_WAVE (T * D * NC + NSRC * T * 64)

extern "C" __global__ __launch_bounds__(64 * NWB) void sig_bwd_lanes(const float* __restrict__ path,
        const float* __restrict__ coeffs, const float* __restrict__ grad, long B, long P, float* gdx)
{
    __shared__ __attribute__((aligned(16))) float smem[NWB * BW_PER_WAVE];
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long wave = (long)blockIdx.x * NWB + wib;
    if (wave >= B * WAVES) return;
    float* Ec = smem + wib * BW_PER_WAVE;
    float* Vb = Ec + T * D * NC;
    const long b = wave / WAVES;
    const int p0 = __builtin_amdgcn_readfirstlane((int)(wave - b * WAVES) * 64);
    const bool valid = p0 + lane < NL;
    const int p = valid ? p0 + lane : NL - 1;
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + b * P * D;
    const long L = P - 1;
    const float* cf = coeffs + b * NWORDS;
    const float* gr = grad + b * NWORDS;

    // signature and adjoints at the end of the path; a word shared by several lanes has its adjoint in the first
    float Sc[K], Ac[K], A1[D];
#pragma unroll
    for (int k = 1; k <= K; ++k) {
        const long w = level_start(k) + p / ipow(D, K - k);
        Sc[k - 1] = cf[w];
        Ac[k - 1] = valid && p % ipow(D, K - k) == 0 ? gr[w] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < D; ++j) A1[j] = valid ? gr[level_start(K + 1) + (long)p * D + j] : 0.0f;
#if R == 2
    float S1[D], An[D][D];
#pragma unroll
    for (int j = 0; j < D; ++j) {
        S1[j] = cf[level_start(K + 1) + (long)p * D + j];
#pragma unroll
        for (int jj = 0; jj < D; ++jj) An[j][jj] = valid ? gr[level_start(K + 2) + ((long)p * D + j) * D + jj] : 0.0f;
    }
#endif

    const long ntiles = (L + T - 1) / T;
    float dxn = fetch_increment(X, (ntiles - 1) * T, L, lane);
    for (long n = ntiles - 1; n >= 0; --n) {
        wave_lds_fence();
        stage_increment(Ec, dxn, lane);
        wave_lds_fence();
        dxn = fetch_increment(X, (n - 1) * T, L, lane);
#pragma unroll 2
        for (int tt = T - 1; tt >= 0; --tt) {
            const float* Et = Ec + tt * D * NC;
            float ec[K][NC];
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float* src = Et + letter[k] * NC;
#pragma unroll
                for (int t = 0; t <= N - (k + 1); ++t) ec[k][t] = src[t];
            }
            // reconstruction with -dX, then the Horner intermediates with +dX from the reconstructed signature
            float am[K + 1][N + 2], ap[K + 1][N + 2];
#pragma unroll
            for (int t = 0; t < N + 2; ++t) am[0][t] = ap[0][t] = 1.0f;
#pragma unroll
            for (int k = 1; k <= K; ++k) {
#pragma unroll
                for (int t = 1; t <= N - k; ++t) am[k][t] = __builtin_fmaf(-ec[k - 1][t], am[k - 1][t + 1], Sc[k - 1]);
                Sc[k - 1] = __builtin_fmaf(-ec[k - 1][0], am[k - 1][1], Sc[k - 1]);
#pragma unroll
                for (int t = 1; t <= N - k; ++t) ap[k][t] = __builtin_fmaf(ec[k - 1][t], ap[k - 1][t + 1], Sc[k - 1]);
            }
            float* vb = Vb + tt * 64 + lane;
            float gb[K + 1][N + 2];
#pragma unroll
            for (int k = 0; k <= K; ++k)
#pragma unroll
                for (int t = 0; t < N + 2; ++t) gb[k][t] = 0.0f;
            float g1 = 0.0f;
#if R == 1
            // the leaves: constant adjoints
#pragma unroll
            for (int j = 0; j < D; ++j) {
                vb[j * T * 64] = A1[j] * ap[K][1];
                g1 = __builtin_fmaf(Et[j * NC], A1[j], g1);
            }
#else
            float y[D];
#pragma unroll
            for (int j = 0; j < D; ++j) y[j] = 0.0f;
            const float hp2 = 0.5f * ap[K][2];
            float g2 = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) {
                S1[j] = __builtin_fmaf(-Et[j * NC], am[K][1], S1[j]);
                const float Gp = __builtin_fmaf(Et[j * NC + 1], ap[K][2], S1[j]);
                float h = 0.0f;
#pragma unroll
                for (int jj = 0; jj < D; ++jj) {
                    h = __builtin_fmaf(Et[jj * NC], An[j][jj], h);
                    y[jj] = __builtin_fmaf(An[j][jj], Gp, y[jj]);
                }
                const float q0 = A1[j];
                A1[j] = q0 + h;
                y[j] = __builtin_fmaf(q0, ap[K][1], y[j]);
                y[j] = __builtin_fmaf(h, hp2, y[j]);
                g1 = __builtin_fmaf(Et[j * NC], q0, g1);
                g2 = __builtin_fmaf(Et[j * NC + 1], h, g2);
            }
            gb[K][2] = g2;
#pragma unroll
            for (int j = 0; j < D; ++j) vb[j * T * 64] = y[j];
#endif
            gb[K][1] = g1;
            // the chain
#pragma unroll
            for (int k = K; k >= 1; --k) {
                gb[k][0] = Ac[k - 1];
                float gc = 0.0f, asum = 0.0f;
#pragma unroll
                for (int t = 0; t <= N - k; ++t) {
                    const float q = gb[k][t];
                    asum += q;
                    gc = __builtin_fmaf(q * inv1(t), ap[k - 1][t + 1], gc);
                    gb[k - 1][t + 1] = __builtin_fmaf(ec[k - 1][t], q, gb[k - 1][t + 1]);
                }
                Ac[k - 1] = asum;
                vb[(D + k - 1) * T * 64] = gc;
            }
        }
        wave_lds_fence();
        if (lane < T * D) {
            const int j = lane / T, t = lane % T;
            // rows of the letters below u: all 64 lanes.  The rows lie 256 bytes apart, so every lane starts at
            // another 16-byte piece of its row.
            const f4* row = (const f4*)(Vb + lane * 64);
            f4 acc4 = row[lane & 15];
#pragma unroll
            for (int i = 1; i < 16; ++i) acc4 += row[(i + lane) & 15];
            float acc = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
            // chain position k: the lanes whose k-th letter is j, runs of D^(K-k) words every D^(K-k+1)
#pragma unroll
            for (int k = 1; k <= K; ++k) {
                const int s = ipow(D, K - k), period = s * D;
                const float* V = Vb + ((D + k - 1) * T + t) * 64;
                for (int rs = (p0 / period) * period + j * s; rs < p0 + 64; rs += period) {
                    const int lo = rs > p0 ? rs : p0;
                    const int hi = rs + s < p0 + 64 ? rs + s : p0 + 64;
                    for (int q = lo; q < hi; ++q) acc += V[q - p0];
                }
            }
            const long sg = n * T + t;
            if (sg < L) __hip_atomic_fetch_add(gdx + (b * L + sg) * D + j, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}
#endif
)SRC";

}  // namespace

LanesShape lanes_shape(int d, int depth)
{
    LanesShape s{};
    if (d < 2 || d > 64 || depth < 2 || depth > 12) return s;
    // two levels per lane while their state fits the registers (forward d + d^2 values, backward about twice that)
    s.R = (d <= 8 && depth >= 3) ? 2 : 1;
    s.T = 64 / d < 8 ? 64 / d : 8;
    double lanes = 1.0;
    for (int k = 0; k < depth - s.R; ++k) lanes *= d;
    if (lanes > 1.0e9) return LanesShape{};
    s.lanes = (int64_t)lanes;
    s.waves = (s.lanes + 63) / 64;
    const int NC = (depth + 3) / 4 * 4;
    const size_t per_wave = ((size_t)s.T * d * NC + (size_t)(d + depth - s.R) * s.T * 64) * sizeof(float);
    s.nwb = (int)(per_wave * 4 <= 64 * 1024 ? 4 : (per_wave * 2 <= 64 * 1024 ? 2 : (per_wave <= 64 * 1024 ? 1 : 0)));
    s.ok = s.nwb > 0;
    return s;
}

std::string lanes_source(int d, int depth, const LanesShape& s, bool backward)
{
    std::ostringstream o;
    o << "#define D " << d << "\n#define N " << depth << "\n#define R " << s.R << "\n#define T " << s.T << "\n#define NWB "
      << s.nwb << "\n#define BACKWARD " << (backward ? 1 : 0) << "\n"
      << kLanesSource;
    return o.str();
}

}  // namespace sig
