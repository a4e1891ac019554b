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
#include <algorithm>
#include <sstream>
#include <string>

#include "jit.hpp"

namespace sig {
namespace {

const char* const kLanesSource = R"SRC(
#define K (N - R)
#define NC ((N + 3) / 4 * 4)
#define DP ((D + 3) / 4 * 4)
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
// chain positions k = 1 .. NU whose letter takes at most three values inside a wavefront (runs of D^(K-k) >= 32 lanes)
constexpr int count_wide()
{
    int n = 0;
    for (int k = 1; k <= K; ++k) n += ipow(D, K - k) >= 32 ? 1 : 0;
    return n;
}

#define NL ipow(D, K)                       /* words of length K = lanes per path */
#define WAVES ((NL + 63) / 64)
#define NWORDS (level_start(N) + ipow(D, N))
#define NU count_wide()

static_assert(K >= 1 && (R == 1 || R == 2), "a lane holds a word of length N - R and one or two levels below it");
static_assert(T * D <= 64 && TS % T == 0, "one lane per (letter, segment) of a tile; whole tiles per staging tile");

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Increments are staged TS segments at a time (a multiple of T; the global loads of the next staging tile are in
// flight while this one is worked on, and a longer tile hides their latency when a SIMD has a single wavefront).
// Element e = lane + 64 q of a staging tile is (segment j0 + e / D, letter e % D); zero outside [0, L).
#define EPL ((TS * D + 63) / 64)
__device__ __forceinline__ void fetch_increments(const float* __restrict__ X, long j0, long L, int lane, float (&dx)[EPL])
{
    // points are rows of D floats, so element e of the tile is X[j0 D + e + D] - X[j0 D + e]
    const long base = j0 * D, lim = L * D;
#pragma unroll
    for (int q = 0; q < EPL; ++q) {
        long idx = base + lane + 64 * q;
        const bool ok = idx >= 0 && idx < lim;
        idx = idx < 0 ? 0 : (idx < lim ? idx : lim - 1);
        const float x1 = X[idx + D], x0 = X[idx];
        dx[q] = ok ? x1 - x0 : 0.0f;
    }
}
// LDS of a staging tile: Ec[segment][letter][t] = dX / (t + 1) for the chain (a lane reads the row of its own
// letter), and E0[segment][letter] = dX, E1 = dX / 2 as contiguous rows for the levels below u (every lane reads all
// letters)
#define TILE_F (TS * D * NC + 2 * TS * DP)
__device__ __forceinline__ void stage_increments(float* Ec, const float (&dx)[EPL], int lane)
{
#pragma unroll
    for (int q = 0; q < EPL; ++q) {
        const int e = lane + 64 * q;
        if (e < TS * D) {
#pragma unroll
            for (int t = 0; t < N; ++t) Ec[e * NC + t] = dx[q] * inv1(t);
            float* E0 = Ec + TS * D * NC;
            E0[(e / D) * DP + e % D] = dx[q];
            E0[TS * DP + (e / D) * DP + e % D] = dx[q] * 0.5f;
        }
    }
}
// the D increments of a segment from one of the contiguous rows
__device__ __forceinline__ void load_row(const float* row, float (&e)[DP])
{
#pragma unroll
    for (int q = 0; q < DP / 4; ++q) {
        const f4 v = ((const f4*)row)[q];
        e[4 * q] = v[0]; e[4 * q + 1] = v[1]; e[4 * q + 2] = v[2]; e[4 * q + 3] = v[3];
    }
}

// Row r: a whole path (win == nullptr: path r) or window r % KW of path r / KW, between the points win[2 k] and
// win[2 k + 1] clamped to the path, at most max_len segments; read straight from the path.
__device__ __forceinline__ void row_of(const long* __restrict__ win, long KW, long max_len, long r, long P, long& b, long& first,
                                       long& L)
{
    if (win == nullptr) {
        b = r;
        first = 0;
        L = P - 1;
    } else {
        b = r / KW;
        const long k = r - b * KW;
        long l = win[2 * k], e = win[2 * k + 1];
        l = l < 0 ? 0 : (l > P - 1 ? P - 1 : l);
        e = e < l ? l : (e > P - 1 ? P - 1 : e);
        first = l;
        L = e - l < max_len ? e - l : max_len;
    }
}

#if !BACKWARD
extern "C" __global__ __launch_bounds__(64 * NWB) void sig_fwd_lanes(const float* __restrict__ path, long B, long P,
                                                                      float* __restrict__ coeffs, const long* __restrict__ win,
                                                                      long KW, long max_len)
{
    __shared__ __attribute__((aligned(16))) float smem[NWB * TILE_F];
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long wave = (long)blockIdx.x * NWB + wib;
    if (wave >= B * (win ? KW : 1) * WAVES) return;      // wavefronts share nothing: no barrier is skipped
    float* Ec = smem + wib * TILE_F;
    const float* E0 = Ec + TS * D * NC;
    const long row = wave / WAVES;
    long b, first, L;
    row_of(win, KW, max_len, row, P, b, first, L);
    const int p0 = __builtin_amdgcn_readfirstlane((int)(wave - row * WAVES) * 64);
    const bool valid = p0 + lane < NL;
    const int p = valid ? p0 + lane : NL - 1;
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    const float* X = path + (b * P + first) * D;

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

    const long ntiles = (L + TS - 1) / TS;
    float dxn[EPL];
#pragma unroll
    for (int q = 0; q < EPL; ++q) dxn[q] = 0.0f;
    if (L > 0) fetch_increments(X, 0, L, lane, dxn);     // an empty window reads nothing and stores the zero signature
    for (long n = 0; n < ntiles; ++n) {
        wave_lds_fence();
        stage_increments(Ec, dxn, lane);
        wave_lds_fence();
        fetch_increments(X, (n + 1) * TS, L, lane, dxn); // past the end: zeros, and a zero increment changes nothing
#pragma unroll 2
        for (int tt = 0; tt < TS; ++tt) {
            const float* Et = Ec + tt * D * NC;
            float e0[DP];
            load_row(E0 + tt * DP, e0);
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
#if R == 2
            float e1[DP];
            load_row(E0 + TS * DP + tt * DP, e1);
#endif
#pragma unroll
            for (int j = 0; j < D; ++j) {
#if R == 2
                const float Gp = __builtin_fmaf(e1[j], ap[K][2], S1[j]);
#pragma unroll
                for (int jj = 0; jj < D; ++jj) S2[j][jj] = __builtin_fmaf(e0[jj], Gp, S2[j][jj]);
#endif
                S1[j] = __builtin_fmaf(e0[j], ap[K][1], S1[j]);
            }
        }
    }

    if (!valid) return;
    float* out = coeffs + row * NWORDS;
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
// per chain position (to the lane's own letter at that position).  They go to LDS rows [source][segment][lane] for
// the segments of a tile and are summed per tile:
//   - rows of the letters below u: lane j T + t adds up row (j, t);
//   - chain positions whose letter runs over fewer than 32 lanes: the same lane adds the members of its letter;
//   - chain positions with longer runs (at most three of them reach into a wavefront): a lane writes to the row of
//     its run, and these rows are summed like the rows of the first kind by a second group of lanes;
// every total goes to gdx (zeroed by the caller) with one floating-point atomic.
#define NSRC (D + K + 2 * NU)
#define BW_PER_WAVE (TILE_F + NSRC * T * 64)
// row of chain position k (1-based): three rows for each of the first NU positions, one for the others
constexpr int chain_row(int k) { return k <= NU ? D + 3 * (k - 1) : D + 3 * NU + (k - NU - 1); }

__device__ __forceinline__ float row_sum(const float* row, int lane)
{
    // rows lie 256 bytes apart: every lane starts at another 16-byte piece of its row
    const f4* r = (const f4*)row;
    f4 acc = r[lane & 15];
#pragma unroll
    for (int i = 1; i < 16; ++i) acc += r[(i + lane) & 15];
    return (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

extern "C" __global__ __launch_bounds__(64 * NWB) void sig_bwd_lanes(const float* __restrict__ path,
        const float* __restrict__ coeffs, const float* __restrict__ grad, long B, long P, float* gdx,
        const long* __restrict__ win, long KW, long max_len)
{
    __shared__ __attribute__((aligned(16))) float smem[NWB * BW_PER_WAVE];
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long wave = (long)blockIdx.x * NWB + wib;
    if (wave >= B * (win ? KW : 1) * WAVES) return;
    float* Ec = smem + wib * BW_PER_WAVE;
    const float* E0 = Ec + TS * D * NC;
    float* Vb = Ec + TILE_F;
    const long row = wave / WAVES;
    long b, first, L;
    row_of(win, KW, max_len, row, P, b, first, L);
    const int p0 = __builtin_amdgcn_readfirstlane((int)(wave - row * WAVES) * 64);
    const bool valid = p0 + lane < NL;
    const int p = valid ? p0 + lane : NL - 1;
    int letter[K];
    {
        int q = p;
#pragma unroll
        for (int k = K - 1; k >= 0; --k) { letter[k] = q % D; q /= D; }
    }
    if (L <= 0) return;                                  // an empty window: no gradient (wavefronts share no barrier)
    const float* X = path + (b * P + first) * D;
    const float* cf = coeffs + row * NWORDS;
    const float* gr = grad + row * NWORDS;
    float* const gdx_row = gdx + (b * (P - 1) + first) * D;     // the gradients of overlapping windows add up here

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
    // chain positions with long runs: the run of this lane among those that reach into the wavefront (0, 1 or 2),
    // how many do, and the letter of the first
    int my_run[NU + 1], runs[NU + 1], first_letter[NU + 1];
#pragma unroll
    for (int k = 1; k <= NU; ++k) {
        const int s = ipow(D, K - k);
        my_run[k] = (p0 + lane) / s - p0 / s;
        runs[k] = (p0 + 63) / s - p0 / s + 1;
        first_letter[k] = (p0 / s) % D;
    }

    const long nstage = (L + TS - 1) / TS;
    float dxn[EPL];
    fetch_increments(X, (nstage - 1) * TS, L, lane, dxn);
    for (long ns = nstage - 1; ns >= 0; --ns) {
        wave_lds_fence();
        stage_increments(Ec, dxn, lane);
        wave_lds_fence();
        fetch_increments(X, (ns - 1) * TS, L, lane, dxn);
      for (int sub = TS / T - 1; sub >= 0; --sub) {          // tiles of T segments: the unit of the gradient sums
        const long n = ns * (TS / T) + sub;
#pragma unroll 2
        for (int tt = T - 1; tt >= 0; --tt) {
            const float* Et = Ec + (sub * T + tt) * D * NC;
            float e0[DP];
            load_row(E0 + (sub * T + tt) * DP, e0);
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
                g1 = __builtin_fmaf(e0[j], A1[j], g1);
            }
#else
            float e1[DP];
            load_row(E0 + TS * DP + (sub * T + tt) * DP, e1);
            float y[D];
#pragma unroll
            for (int j = 0; j < D; ++j) y[j] = 0.0f;
            const float hp2 = 0.5f * ap[K][2];
            float g2 = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) {
                S1[j] = __builtin_fmaf(-e0[j], am[K][1], S1[j]);
                const float Gp = __builtin_fmaf(e1[j], ap[K][2], S1[j]);
                float h = 0.0f;
#pragma unroll
                for (int jj = 0; jj < D; ++jj) {
                    h = __builtin_fmaf(e0[jj], An[j][jj], h);
                    y[jj] = __builtin_fmaf(An[j][jj], Gp, y[jj]);
                }
                const float q0 = A1[j];
                A1[j] = q0 + h;
                y[j] = __builtin_fmaf(q0, ap[K][1], y[j]);
                y[j] = __builtin_fmaf(h, hp2, y[j]);
                g1 = __builtin_fmaf(e0[j], q0, g1);
                g2 = __builtin_fmaf(e1[j], h, g2);
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
                if (k <= NU) {
                    const int kk = k <= NU ? k : 0;
                    vb[chain_row(k) * T * 64] = my_run[kk] == 0 ? gc : 0.0f;
                    if (runs[kk] > 1) vb[(chain_row(k) + 1) * T * 64] = my_run[kk] == 1 ? gc : 0.0f;
                    if (runs[kk] > 2) vb[(chain_row(k) + 2) * T * 64] = my_run[kk] == 2 ? gc : 0.0f;
                } else {
                    vb[chain_row(k) * T * 64] = gc;
                }
            }
        }
        wave_lds_fence();
        if (lane < T * D) {
            const int j = lane / T, t = lane % T;
            float acc = row_sum(Vb + lane * 64, lane);
            // chain position k with runs of s < 32 lanes: the lanes whose k-th letter is j, s of them every s D
#pragma unroll
            for (int k = NU + 1; k <= K; ++k) {
                const int s = ipow(D, K - k), period = s * D;
                const float* V = Vb + (chain_row(k) * T + t) * 64;
                const int rs0 = (p0 / period) * period + j * s - p0;     // first run that can reach this wavefront
#pragma unroll
                for (int r = 0; r < (64 + period - 1) / period + 1; ++r)
#pragma unroll
                    for (int u = 0; u < s; ++u) {
                        const int q = rs0 + r * period + u;
                        const bool in = q >= 0 && q < 64;
                        const float v = V[in ? q : 0];
                        acc += in ? v : 0.0f;
                    }
            }
            const long sg = n * T + t;
            if (sg < L) __hip_atomic_fetch_add(gdx_row + sg * D + j, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int base = 0; base < 3 * NU * T; base += 64) {
            const int o = base + lane;
            if (o < 3 * NU * T) {
                const int r = o / T, t = o % T;                           // row D + r: position r / 3 + 1, run r % 3
                int nr = 0, fl = 0;
#pragma unroll
                for (int k = 1; k <= NU; ++k)
                    if (r / 3 + 1 == k) { nr = runs[k]; fl = first_letter[k]; }
                const long sg = n * T + t;
                if (sg < L && r % 3 < nr) {
                    const float acc = row_sum(Vb + ((D + r) * T + t) * 64, lane);
                    const int j = (fl + r % 3) % D;
                    __hip_atomic_fetch_add(gdx_row + sg * D + j, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        wave_lds_fence();                                      // the rows are rewritten by the next tile
      }
    }
}
#endif
)SRC";

}  // namespace

LanesShape lanes_shape(int d, int depth, bool backward, int64_t B, int levels)
{
    LanesShape best{};
    if (d < 2 || d > 64 || depth < 2 || depth > 12) return best;
    const int NC = (depth + 3) / 4 * 4, DP = (d + 3) / 4 * 4;
    double best_cost = 0.0;
    // Two levels per lane while their state fits the registers (forward d + d^2 values, backward twice that and the
    // per-letter sums).  Between the admissible forms: the time of a segment is the instructions of a lane times the
    // wavefronts a SIMD has to run one after the other (1,024 SIMDs); two levels per lane share more work between
    // words but leave few wavefronts for small batches, where one level per lane then has the shorter segment.
    for (int R = 1; R <= 2; ++R) {
        if (levels != 0 && R != levels) continue;
        if (depth - R < 1) continue;
        if (R == 2 && d > (backward ? 10 : 12)) continue;
        LanesShape s{};
        s.R = R;
        s.T = 64 / d < 8 ? 64 / d : 8;
        const int K = depth - R;
        double lanes = 1.0;
        for (int k = 0; k < K; ++k) lanes *= d;
        if (lanes > 1.0e9) continue;
        s.lanes = (int64_t)lanes;
        s.waves = (s.lanes + 63) / 64;
        int chain = 0, wide = 0;
        double run = lanes;
        for (int k = 1; k <= K; ++k) {
            chain += depth - k + 1;
            run /= d;                                      // d^(K - k)
            wide += run >= 32.0 ? 1 : 0;
        }
        const double per_lane = 2.0 * chain + (R == 2 ? (double)d * d + 3.0 * d : 2.0 * d);
        const double rounds = (double)std::max<int64_t>(B, 1) * (double)s.waves / 1024.0;
        const double cost = per_lane * (rounds < 1.0 ? 1.0 : rounds);
        // LDS of a wavefront: the increments of a staging tile and, backward, the gradient rows of the segments of a
        // tile; eight wavefronts of 20 KB fit a compute unit, so longer tiles are cut down to that.  The staging
        // tile is as many tiles as fit (up to 32 segments and three increments per lane): its global loads are issued
        // one staging tile ahead.
        auto lds_bytes = [&](int T, int TS) {
            const size_t tile = (size_t)TS * ((size_t)d * NC + 2 * (size_t)DP);
            return (tile + (backward ? (size_t)(d + K + 2 * wide) * T * 64 : 0)) * sizeof(float);
        };
        // (a lane carries its share of the next staging tile in registers: one increment where the state of two
        // levels already fills them)
        const int staged = (R == 2 && d * d + d > 48) ? 64 : 192;
        if (backward) {
            while (s.T > 1 && lds_bytes(s.T, s.T) > 20 * 1024) --s.T;
            s.TS = s.T;
            while (s.TS + s.T <= 32 && (s.TS + s.T) * d <= staged && lds_bytes(s.T, s.TS + s.T) <= 20 * 1024) s.TS += s.T;
        } else {
            s.T = 1;                                       // no gradient tiles: only the staging tile matters
            s.TS = 32;
            while (s.TS > 2 && (s.TS * d > staged || s.TS % 2 != 0 || lds_bytes(1, s.TS) > 8 * 1024)) --s.TS;
            if (s.TS * d > 64 && s.TS * d > staged) s.TS = 1;
        }
        const size_t per_wave = lds_bytes(s.T, s.TS);
        s.nwb = (int)(per_wave * 4 <= 64 * 1024 ? 4 : (per_wave * 2 <= 64 * 1024 ? 2 : (per_wave <= 64 * 1024 ? 1 : 0)));
        s.ok = s.nwb > 0;
        if (s.ok && (!best.ok || cost < best_cost)) {
            best = s;
            best_cost = cost;
        }
    }
    return best;
}

std::string lanes_source(int d, int depth, const LanesShape& s, bool backward)
{
    std::ostringstream o;
    o << "#define D " << d << "\n#define N " << depth << "\n#define R " << s.R << "\n#define T " << s.T << "\n#define TS " << s.TS << "\n#define NWB "
      << s.nwb << "\n#define BACKWARD " << (backward ? 1 : 0) << "\n"
      << kLanesSource;
    return o.str();
}

}  // namespace sig
