// Table-driven signature kernels for arbitrary prefix-closed word sets (gfx950).
//
// Mapping: one wavefront = one work unit (a piece of the word tree, see wordset.hpp) x 64 paths,
// lane = path.  The unit's program is wave-uniform, so its words are decoded by the scalar unit and
// every vector instruction is a lane-private multiply-add.  Coefficients live in LDS as
// [word][lane] rows (conflict-free, lane-private), the Horner chain of the current root-to-node walk
// lives in registers with compile-time indices (one switch case per word length).
//
// Forward step for a word u of length k inside a unit (Algorithm 1 with the intermediates of words
// that share a prefix computed once):   for t = 0..h(u)
//     A_k[t] = S(u) + dX^{(u_k)}/(t+1) * A_{k-1}[t+1],      A_0[.] = 1,
// where A_k[t] is the Horner accumulator "S(w_[k]) + h" of Algorithm 1 for target words of length
// k + t that pass through u; t = 0 gives the new S(u).
//
// Backward step (Section 4): S_{0,t_{j-1}} is reconstructed from S_{0,t_j} with the same recursion
// and -dX (Proposition 4.6); the accumulators are recomputed with +dX and the recursion is run in
// reverse for the adjoint, which carries the right factors of Proposition 4.1 aggregated over all
// words with a common prefix.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/sig.h"
#include "kernels.hpp"

#include <cstdlib>

// Workspace of sig_backward_static, the entry point for callers that cannot allocate: one copy per device, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress (static_scratch below); kernels
// and fills receive the address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[SIG_STATIC_SCRATCH_BYTES];

namespace sig {

namespace {

constexpr int kWave = 64;
constexpr size_t kMaxLds = 160 * 1024;   // LDS per compute unit on gfx950

__device__ __forceinline__ float inv_of(int t)   // 1 / (t + 1)
{
    constexpr float tab[16] = {1.0f,        1.0f / 2.0f,  1.0f / 3.0f,  1.0f / 4.0f,  1.0f / 5.0f,  1.0f / 6.0f,
                               1.0f / 7.0f, 1.0f / 8.0f,  1.0f / 9.0f,  1.0f / 10.0f, 1.0f / 11.0f, 1.0f / 12.0f,
                               1.0f / 13.0f, 1.0f / 14.0f, 1.0f / 15.0f, 1.0f / 16.0f};
    return tab[t];
}

// Register file of Horner accumulators: a[k][t], k = word length, t = extra target length.
template <int MAXK>
struct Chain {
    float a[MAXK + 1][MAXK + 2];
};

template <int MAXK, int K>
__device__ __forceinline__ float fwd_node(Chain<MAXK>& A, float dxl, float s, int h)
{
    // t >= 1 first (they read the old S), then t = 0 which is the new S
#pragma unroll
    for (int t = 1; t <= MAXK - K; ++t)
        if (t <= h) A.a[K][t] = fmaf(dxl * inv_of(t), A.a[K - 1][t + 1], s);
    const float snew = fmaf(dxl, A.a[K - 1][1], s);
    A.a[K][0] = snew;
    return snew;
}

template <int MAXK, int K>
struct FwdDispatch {
    static __device__ __forceinline__ float run(Chain<MAXK>& A, int level, float dxl, float s, int h)
    {
        if (level == K) return fwd_node<MAXK, K>(A, dxl, s, h);
        if constexpr (K < MAXK) return FwdDispatch<MAXK, K + 1>::run(A, level, dxl, s, h);
        return s;
    }
};

template <int MAXK>
__global__ __launch_bounds__(kWave) void fwd_generic_kernel(const UnitDesc* __restrict__ units,
                                                            const uint32_t* __restrict__ ops,
                                                            const int32_t* __restrict__ slot_word,
                                                            const float* __restrict__ path, int64_t B, int64_t P, int d,
                                                            int64_t nW, float* __restrict__ coeffs)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x;
    const UnitDesc ud = units[blockIdx.x];
    const int64_t b = (int64_t)blockIdx.y * kWave + lane;
    const bool valid = b < B;
    const float* X = path + (valid ? b : B - 1) * P * d;
    float* dx = lds;                    // [d][64]
    float* S = lds + (size_t)d * kWave;   // [n_slots][64]
    for (int s = 0; s < ud.n_slots; ++s) S[s * kWave + lane] = 0.0f;

    Chain<MAXK> A;
#pragma unroll
    for (int t = 0; t < MAXK + 2; ++t) A.a[0][t] = 1.0f;

    const uint32_t* prog = ops + ud.op_off;
    for (int64_t j = 1; j < P; ++j) {
        for (int i = 0; i < d; ++i) dx[i * kWave + lane] = X[j * d + i] - X[(j - 1) * d + i];
        for (int o = 0; o < ud.n_ops; ++o) {
            const uint32_t op = prog[o];
            const int letter = op & 0xfff, level = (op >> 12) & 0xf, h = (op >> 16) & 0xf;
            const float dxl = dx[letter * kWave + lane];
            const float s = S[o * kWave + lane];
            S[o * kWave + lane] = FwdDispatch<MAXK, 1>::run(A, level, dxl, s, h);
        }
    }
    if (valid) {
        const int32_t* sw = slot_word + ud.slot_off;
        for (int s = 0; s < ud.n_slots; ++s) {
            const int32_t w = sw[s];
            if (w >= 0) coeffs[b * nW + w] = S[s * kWave + lane];
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// backward

template <int MAXK>
struct BwdRegs {
    float am[MAXK + 1][MAXK + 2];   // accumulators with -dX (reconstruction)
    float ap[MAXK + 1][MAXK + 2];   // accumulators with +dX, from the reconstructed S_{0,t_{j-1}}
    float gb[MAXK + 1][MAXK + 2];   // adjoints of ap
    int slot[MAXK + 1];             // LDS row of the open word at each length
};

template <int MAXK, int K>
__device__ __forceinline__ void bwd_leaf(BwdRegs<MAXK>& R, float dxl, float* S, const float* Ab, float* gc, int row,
                                         int lane, int letter)
{
    const float s = S[row * kWave + lane];
    const float a = Ab[row * kWave + lane];
    S[row * kWave + lane] = fmaf(-dxl, R.am[K - 1][1], s);
    gc[letter * (kWave + 1) + lane] = fmaf(a, R.ap[K - 1][1], gc[letter * (kWave + 1) + lane]);
    R.gb[K - 1][1] = fmaf(dxl, a, R.gb[K - 1][1]);
}

template <int MAXK, int K>
__device__ __forceinline__ void bwd_enter(BwdRegs<MAXK>& R, float dxl, float* S, int row, int lane, int h)
{
    const float s = S[row * kWave + lane];
#pragma unroll
    for (int t = 1; t <= MAXK - K; ++t)
        if (t <= h) R.am[K][t] = fmaf(-dxl * inv_of(t), R.am[K - 1][t + 1], s);
    const float sp = fmaf(-dxl, R.am[K - 1][1], s);
    S[row * kWave + lane] = sp;
#pragma unroll
    for (int t = 1; t <= MAXK - K; ++t)
        if (t <= h) {
            R.ap[K][t] = fmaf(dxl * inv_of(t), R.ap[K - 1][t + 1], sp);
            R.gb[K][t] = 0.0f;
        }
    R.slot[K] = row;
}

template <int MAXK, int K>
__device__ __forceinline__ void bwd_leave(BwdRegs<MAXK>& R, float dxl, float* Ab, float* gc, int lane, int letter, int h)
{
    const int row = R.slot[K];
    const float a = Ab[row * kWave + lane];
    float asum = a;
    float gsum = a * R.ap[K - 1][1];
    R.gb[K - 1][1] = fmaf(dxl, a, R.gb[K - 1][1]);
#pragma unroll
    for (int t = 1; t <= MAXK - K; ++t)
        if (t <= h) {
            const float g = R.gb[K][t];
            asum += g;
            gsum = fmaf(g * inv_of(t), R.ap[K - 1][t + 1], gsum);
            R.gb[K - 1][t + 1] = fmaf(dxl * inv_of(t), g, R.gb[K - 1][t + 1]);
        }
    Ab[row * kWave + lane] = asum;
    gc[letter * (kWave + 1) + lane] += gsum;
}

template <int MAXK, int K>
struct BwdDispatch {
    static __device__ __forceinline__ void run(BwdRegs<MAXK>& R, int level, int kind, float dxl, float* S, float* Ab,
                                               float* gc, int row, int lane, int letter, int h)
    {
        if (level == K) {
            if (kind == OP_LEAF) bwd_leaf<MAXK, K>(R, dxl, S, Ab, gc, row, lane, letter);
            else if (kind == OP_ENTER) bwd_enter<MAXK, K>(R, dxl, S, row, lane, h);
            else bwd_leave<MAXK, K>(R, dxl, Ab, gc, lane, letter, h);
            return;
        }
        if constexpr (K < MAXK) BwdDispatch<MAXK, K + 1>::run(R, level, kind, dxl, S, Ab, gc, row, lane, letter, h);
    }
};

// gdx: [B][L][d] partial sums of dLoss/d dX, zeroed before the launch; units add into it.
template <int MAXK>
__global__ __launch_bounds__(kWave) void bwd_generic_kernel(const UnitDesc* __restrict__ units,
                                                            const uint32_t* __restrict__ ops,
                                                            const int32_t* __restrict__ slot_word,
                                                            const float* __restrict__ path,
                                                            const float* __restrict__ coeffs,
                                                            const float* __restrict__ grad_coeffs, int64_t B, int64_t P,
                                                            int d, int64_t nW, int tile_steps, float* gdx)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x;
    const UnitDesc ud = units[blockIdx.x];
    const int64_t b0 = (int64_t)blockIdx.y * kWave;
    const int64_t b = b0 + lane;
    const bool valid = b < B;
    const int64_t bc = valid ? b : B - 1;
    const float* X = path + bc * P * d;
    const int64_t L = P - 1;
    float* dx = lds;                                          // [d][64]
    float* S = dx + (size_t)d * kWave;                         // [n_slots][64]
    float* Ab = S + (size_t)ud.n_slots * kWave;                // [n_slots][64]
    float* gt = Ab + (size_t)ud.n_slots * kWave;               // [tile_steps * d][65]
    {
        const int32_t* sw = slot_word + ud.slot_off;
        for (int s = 0; s < ud.n_slots; ++s) {
            const int32_t w = sw[s];
            const int32_t wi = w >= 0 ? w : ~w;
            S[s * kWave + lane] = coeffs[bc * nW + wi];
            Ab[s * kWave + lane] = w >= 0 ? grad_coeffs[bc * nW + wi] : 0.0f;
        }
    }
    BwdRegs<MAXK> R;
#pragma unroll
    for (int t = 0; t < MAXK + 2; ++t) {
        R.am[0][t] = 1.0f;
        R.ap[0][t] = 1.0f;
        R.gb[0][t] = 0.0f;
    }
    const uint32_t* prog = ops + ud.op_off;
    const int nvalid = (int)((B - b0) < kWave ? (B - b0) : kWave);
    for (int64_t st = L - 1; st >= 0; --st) {          // st = j - 1, segment j runs from point st to st + 1
        const int tt = (int)(st % tile_steps);
        float* gc = gt + (size_t)tt * d * (kWave + 1);
        for (int i = 0; i < d; ++i) {
            dx[i * kWave + lane] = X[(st + 1) * d + i] - X[st * d + i];
            gc[i * (kWave + 1) + lane] = 0.0f;
        }
        int row = 0;
        for (int o = 0; o < ud.n_ops; ++o) {
            const uint32_t op = prog[o];
            const int letter = op & 0xfff, level = (op >> 12) & 0xf, h = (op >> 16) & 0xf, kind = (op >> 20) & 3;
            const float dxl = dx[letter * kWave + lane];
            BwdDispatch<MAXK, 1>::run(R, level, kind, dxl, S, Ab, gc, row, lane, letter, h);
            row += (kind != OP_LEAVE);
        }
        if (tt == 0) {
            // flush the tile: for each path, (step, letter) is contiguous in gdx.  Lanes now read
            // rows written by other lanes, hence the barriers (the block is one wavefront).
            __syncthreads();
            const int64_t last = st + tile_steps < L ? st + tile_steps : L;
            const int cnt = (int)(last - st) * d;
            for (int bb = 0; bb < nvalid; ++bb) {
                float* dst = gdx + ((b0 + bb) * L + st) * d;
                for (int e = lane; e < cnt; e += kWave) unsafeAtomicAdd(dst + e, gt[e * (kWave + 1) + bb]);
            }
            __syncthreads();
        }
    }
}

// Row r of the specialised kernels: a whole path (no window list: path r, all P - 1 segments), time chunk r % K of path
// r / K (K > 1 without windows: segments from (r % K) max_len on), or window r % K of path r / K, between the points
// win[2 k] and win[2 k + 1] clamped to the path, at most max_len segments.
__device__ __forceinline__ void lane_row(const WindowList& wl, int64_t r, int64_t P, int64_t& b, int64_t& first, int64_t& len)
{
    if (!wl.several_rows()) {
        b = r;
        first = 0;
        len = P - 1;
    } else if (wl.win == nullptr) {                   // time chunk r % K of path r / K
        b = r / wl.K;
        first = (r - b * wl.K) * wl.max_len;
        len = P - 1 - first < wl.max_len ? P - 1 - first : wl.max_len;
        if (len < 0) len = 0;
    } else {
        b = r / wl.K;
        const int64_t k = r - b * wl.K;
        int64_t l = wl.win[2 * k], e = wl.win[2 * k + 1];
        l = l < 0 ? 0 : (l > P - 1 ? P - 1 : l);
        e = e < l ? l : (e > P - 1 ? P - 1 : e);
        first = l;
        len = e - l < wl.max_len ? e - l : wl.max_len;
    }
}

// Increments, differenced and transposed for the run-time specialised kernels (lane = row):
//   dxT[((g * Lpad + j) * d + i) * 64 + lane] = X[b][first + j + 1][i] - X[b][first + j][i],  row 64 g + lane,
// zero for padded segments j >= the row's length and for rows past the last.
// One workgroup takes 64 rows x TS segments: a wavefront reads runs of consecutive floats of its 16 rows
// (coalesced), the differences go to an LDS tile [segment * d + letter][row] and leave it as rows of 64 lanes.
__global__ __launch_bounds__(256) void increments_transposed_kernel(const float* __restrict__ path, int64_t R_rows, int64_t P, int d, int64_t Lpad, int TS,
                                             int64_t tiles, WindowList wl, float* __restrict__ dxT, float* __restrict__ zeroed)
{
    extern __shared__ float tile[];                       // [TS * d][65]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = 4;
    const int64_t g = blockIdx.x / tiles;
    const int64_t j0 = (blockIdx.x % tiles) * TS;
    const int R = TS * d;
    // 16 rows per wavefront (workgroups of 256 threads).  Every load is issued unconditionally, from a clamped
    // address, before the first value is used: behind a branch per row the sixteen round trips to memory would run one
    // after the other.
    for (int e0 = 0; e0 < R; e0 += kWave) {
        const int e = e0 + lane;
        const int64_t seg = j0 + e / d;
        // eight rows at a time (sixteen loads in flight): offsets, values and flags of all sixteen rows at once
        // would not fit the registers of the workgroup
#pragma unroll
        for (int q0 = 0; q0 < 16; q0 += 8) {
            int64_t off[8];
            bool ok[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int64_t r = g * kWave + wave * 16 + q0 + q;
                int64_t b = 0, first = 0, len = 0;
                if (r < R_rows) lane_row(wl, r, P, b, first, len);         // uniform over the wavefront
                ok[q] = e < R && seg < len;                                // then point first + seg + 1 <= P - 1
                off[q] = ok[q] ? (b * P + first + j0) * d + e : 0;         // path[0], path[d] exist: P >= 2
            }
            float hi[8], lo[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                hi[q] = path[off[q] + d];
                lo[q] = path[off[q]];
            }
            if (e < R) {
#pragma unroll
                for (int q = 0; q < 8; ++q) tile[e * 65 + wave * 16 + q0 + q] = ok[q] ? hi[q] - lo[q] : 0.0f;
            }
        }
    }
    __syncthreads();
    const int64_t base = ((g * Lpad + j0) * d) * kWave;
    for (int e = wave; e < R; e += nwaves)
        if (j0 + e / d < Lpad) {
            dxT[base + (int64_t)e * kWave + lane] = tile[e * 65 + lane];
            if (zeroed) zeroed[base + (int64_t)e * kWave + lane] = 0.0f;   // an array of the same layout, cleared on the way
        }
}

__global__ void fill_zero_kernel(float* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// dX_j = X_j - X_{j-1}  =>  dLoss/dX_j = dLoss/d dX_j - dLoss/d dX_{j+1}   (Section 4.1)
__global__ void grad_points_kernel(const float* __restrict__ gdx, int64_t B, int64_t P, int d, float* __restrict__ grad_path)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = B * P * d;
    if (i >= n) return;
    const int64_t c = i % d;
    const int64_t j = (i / d) % P;
    const int64_t b = i / (d * P);
    const int64_t L = P - 1;
    const float here = j >= 1 ? gdx[(b * L + (j - 1)) * d + c] : 0.0f;
    const float next = j < L ? gdx[(b * L + j) * d + c] : 0.0f;
    grad_path[i] = here - next;
}

template <int MAXK>
hipError_t launch_fwd(const GenericArgs& a, hipStream_t stream)
{
    const size_t lds = ((size_t)a.d + (size_t)a.max_slots) * kWave * sizeof(float);
    if (lds > kMaxLds) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_generic_kernel<MAXK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)a.n_units, (unsigned)((a.B + kWave - 1) / kWave));
    fwd_generic_kernel<MAXK><<<grid, kWave, lds, stream>>>(a.units, a.ops, a.slot_word, a.path, a.B, a.P, a.d, a.nW, a.coeffs);
    return hipGetLastError();
}

template <int MAXK>
hipError_t launch_bwd(const GenericArgs& a, hipStream_t stream)
{
    const size_t lds = generic_bwd_lds_bytes(a.d, a.max_slots, a.tile_steps);
    if (lds > kMaxLds) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwd_generic_kernel<MAXK>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)a.n_units, (unsigned)((a.B + kWave - 1) / kWave));
    bwd_generic_kernel<MAXK><<<grid, kWave, lds, stream>>>(a.units, a.ops, a.slot_word, a.path, a.coeffs_in, a.grad_coeffs,
                                                          a.B, a.P, a.d, a.nW, a.tile_steps, a.gdx);
    return hipGetLastError();
}

}  // namespace

size_t generic_bwd_lds_bytes(int d, int max_slots, int tile_steps)
{
    return ((size_t)d * kWave + 2 * (size_t)max_slots * kWave + (size_t)tile_steps * d * (kWave + 1)) * sizeof(float);
}

hipError_t generic_forward(const GenericArgs& a, int max_len, hipStream_t stream)
{
    if (max_len <= 4) return launch_fwd<4>(a, stream);
    if (max_len <= 8) return launch_fwd<8>(a, stream);
    return launch_fwd<12>(a, stream);
}

hipError_t generic_backward(const GenericArgs& a, int max_len, hipStream_t stream)
{
    if (max_len <= 4) return launch_bwd<4>(a, stream);
    if (max_len <= 8) return launch_bwd<8>(a, stream);
    return launch_bwd<12>(a, stream);
}

hipError_t increments_transposed(const float* path, int64_t B, int64_t P, int d, int64_t Lpad, float* dxT, float* zeroed,
                                 hipStream_t stream, const WindowList& wl)
{
    const int64_t rows = B * wl.rows_per_path();
    const int64_t groups = (rows + kWave - 1) / kWave;
    if (groups <= 0 || Lpad <= 0 || d <= 0) return hipSuccess;
    const int TS = std::max(1, 64 / d);
    const size_t lds = (size_t)TS * d * 65 * sizeof(float);
    const int64_t tiles = (Lpad + TS - 1) / TS;
    if (lds > 64 * 1024 || tiles > 0x7fffffff / groups) return hipErrorInvalidValue;
    increments_transposed_kernel<<<(unsigned)(tiles * groups), 256, lds, stream>>>(path, rows, P, d, Lpad, TS, tiles, wl, dxT, zeroed);
    return hipGetLastError();
}

// Chain rule for the specialised kernels, whose increment gradients lie in the layout of their increments,
// g[((grp * Lpad + j) * d + i) * 64 + lane]:  dLoss/dX_j = dLoss/d dX_j - dLoss/d dX_{j+1}  (Section 4.1), written to
// grad_path [B][P][d].  A workgroup takes 64 rows x TS points: rows of 64 lanes in, through an LDS tile
// [(TS + 1) * d][65], runs of consecutive floats of one path out.  With a window list a row is a window of its path:
// its points are those of the path from the window's first point on, and the gradients of overlapping windows are
// added up in grad_path (zeroed by the caller) with floating-point atomics.
__global__ __launch_bounds__(256) void grad_points_transposed_kernel(const float* __restrict__ g, int64_t R_rows, int64_t P, int d, int64_t Lpad, int TS,
                                              int64_t tiles, WindowList wl, float* __restrict__ grad_path)
{
    extern __shared__ float tile[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = 4;
    const int64_t grp = blockIdx.x / tiles;
    const int64_t j0 = (blockIdx.x % tiles) * TS;            // points j0 .. j0 + TS - 1 of every row; tile row r: segment j0 - 1 + r / d
    const int rows = (TS + 1) * d;
    int64_t my_b, my_first, my_len = 0;                      // this lane's row: segments past its length count as zero
    if (grp * kWave + lane < R_rows) lane_row(wl, grp * kWave + lane, P, my_b, my_first, my_len);
    // eight loads in flight per lane, each from a clamped address (every segment below Lpad exists in g)
    for (int r0 = wave; r0 < rows; r0 += nwaves * 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int r = r0 + k * nwaves;
            const int64_t j = j0 - 1 + r / d;
            const int64_t jc = j < 0 ? 0 : (j >= Lpad ? Lpad - 1 : j);
            v[k] = g[((grp * Lpad + jc) * d + r % d) * kWave + lane];
            if (j < 0 || j >= my_len) v[k] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int r = r0 + k * nwaves;
            if (r < rows) tile[r * 65 + lane] = v[k];
        }
    }
    __syncthreads();
    for (int q = 0; q < 16; ++q) {
        const int p = wave * 16 + q;
        const int64_t row = grp * kWave + p;
        if (row >= R_rows) break;
        int64_t b, first, len;
        lane_row(wl, row, P, b, first, len);
        float* out = grad_path + (b * P + first + j0) * d;
        for (int e = lane; e < TS * d; e += kWave) {
            if (j0 + e / d <= len) {                          // the row has len + 1 points
                const float v = tile[e * 65 + p] - tile[(e + d) * 65 + p];
                if (wl.several_rows()) unsafeAtomicAdd(out + e, v);
                else out[e] = v;
            }
        }
    }
}

hipError_t grad_points_transposed(const float* g, int64_t B, int64_t P, int d, int64_t Lpad, float* grad_path, hipStream_t stream,
                                  const WindowList& wl)
{
    const int64_t n_rows = B * wl.rows_per_path();
    const int64_t groups = (n_rows + kWave - 1) / kWave;
    const int64_t points = (wl.several_rows() ? wl.max_len : P - 1) + 1;          // points a row can have
    if (groups <= 0 || points <= 0 || d <= 0) return hipSuccess;
    const int TS = std::max(1, 64 / d);
    const size_t lds = (size_t)(TS + 1) * d * 65 * sizeof(float);
    const int64_t tiles = (points + TS - 1) / TS;
    if (lds > 64 * 1024 || tiles > 0x7fffffff / groups) return hipErrorInvalidValue;
    grad_points_transposed_kernel<<<(unsigned)(tiles * groups), 256, lds, stream>>>(g, n_rows, P, d, Lpad, TS, tiles, wl, grad_path);
    return hipGetLastError();
}

// Lead-lag transform (Section 8): out[b][2k] = (X_k, X_k), out[b][2k+1] = (X_k, X_{k+1}); channels 0..d-1 lag,
// d..2d-1 lead.  out: [B, 2P - 1, 2d].
__global__ void leadlag_kernel(const float* __restrict__ path, int64_t B, int64_t P, int d, float* __restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = B * (2 * P - 1) * 2 * d;
    if (i >= n) return;
    const int c = (int)(i % (2 * d));
    const int64_t m = (i / (2 * d)) % (2 * P - 1);
    const int64_t b = i / (2 * d) / (2 * P - 1);
    const int64_t k = c < d ? m / 2 : (m + 1) / 2;      // lag stays at X_{floor(m/2)}, lead moves on at odd m
    out[i] = path[(b * P + k) * d + (c < d ? c : c - d)];
}
// its adjoint: every point gathers the gradients of its (up to four) copies
__global__ void leadlag_backward_kernel(const float* __restrict__ gout, int64_t B, int64_t P, int d, float* __restrict__ gpath)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = B * P * d;
    if (i >= n) return;
    const int c = (int)(i % d);
    const int64_t k = (i / d) % P;
    const int64_t b = i / d / P;
    const int64_t M2 = 2 * P - 1;
    const float* g = gout + b * M2 * 2 * d;
    float acc = g[(2 * k) * 2 * d + c] + g[(2 * k) * 2 * d + d + c];        // row 2k: lag and lead
    if (2 * k + 1 < M2) acc += g[(2 * k + 1) * 2 * d + c];                      // row 2k+1: lag
    if (k > 0) acc += g[(2 * k - 1) * 2 * d + d + c];                            // row 2k-1: lead
    gpath[i] = acc;
}

hipError_t leadlag(const float* path, int64_t B, int64_t P, int d, float* out, hipStream_t stream)
{
    const int64_t n = B * (2 * P - 1) * 2 * d;
    if (n <= 0) return hipSuccess;
    leadlag_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(path, B, P, d, out);
    return hipGetLastError();
}
hipError_t leadlag_backward(const float* gout, int64_t B, int64_t P, int d, float* gpath, hipStream_t stream)
{
    const int64_t n = B * P * d;
    if (n <= 0) return hipSuccess;
    leadlag_backward_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(gout, B, P, d, gpath);
    return hipGetLastError();
}

// Windows (Section 5): window k of a path covers the points l_k .. r_k (segments l_k .. r_k - 1).  Every (path,
// window) pair becomes a path of its own with n_sub points: sub[b K + k][j] = X[b][min(l_k + j, r_k)] - the tail is
// padded with the last point, i.e. with zero increments, which leave a signature unchanged.
__global__ void window_gather_kernel(const float* __restrict__ path, int64_t B, int64_t P, int d, const int64_t* __restrict__ win,
                                     int64_t K, int64_t n_sub, float* __restrict__ sub)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = B * K * n_sub * d;
    if (i >= n) return;
    const int c = (int)(i % d);
    const int64_t j = (i / d) % n_sub;
    const int64_t row = i / d / n_sub;
    const int64_t b = row / K, k = row - b * K;
    int64_t l = win[2 * k], r = win[2 * k + 1];
    l = l < 0 ? 0 : (l > P - 1 ? P - 1 : l);
    r = r < l ? l : (r > P - 1 ? P - 1 : r);
    const int64_t src = l + j < r ? l + j : r;
    sub[i] = path[(b * P + src) * d + c];
}
// adjoint of the gather: grad_path[b][min(l_k + j, r_k)] += grad_sub[b K + k][j]; grad_path zeroed by the caller
__global__ void window_scatter_kernel(const float* __restrict__ gsub, int64_t B, int64_t P, int d, const int64_t* __restrict__ win,
                                      int64_t K, int64_t n_sub, float* __restrict__ gpath)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n = B * K * n_sub * d;
    if (i >= n) return;
    const int c = (int)(i % d);
    const int64_t j = (i / d) % n_sub;
    const int64_t row = i / d / n_sub;
    const int64_t b = row / K, k = row - b * K;
    int64_t l = win[2 * k], r = win[2 * k + 1];
    l = l < 0 ? 0 : (l > P - 1 ? P - 1 : l);
    r = r < l ? l : (r > P - 1 ? P - 1 : r);
    const int64_t dst = l + j < r ? l + j : r;
    unsafeAtomicAdd(gpath + (b * P + dst) * d + c, gsub[i]);
}

hipError_t window_gather(const float* path, int64_t B, int64_t P, int d, const int64_t* win, int64_t K, int64_t n_sub, float* sub,
                         hipStream_t stream)
{
    const int64_t n = B * K * n_sub * d;
    if (n <= 0) return hipSuccess;
    window_gather_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(path, B, P, d, win, K, n_sub, sub);
    return hipGetLastError();
}
hipError_t window_scatter(const float* gsub, int64_t B, int64_t P, int d, const int64_t* win, int64_t K, int64_t n_sub,
                          float* gpath, hipStream_t stream)
{
    const int64_t n = B * K * n_sub * d;
    if (n <= 0) return hipSuccess;
    window_scatter_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(gsub, B, P, d, win, K, n_sub, gpath);
    return hipGetLastError();
}

// ---- log-signature in Lyndon-word coordinates (Section 3.3): the coefficient of the Lyndon word w in the tensor
// logarithm log(1 + x) = sum_k (-1)^{k+1} x^k / k of the signature, where (x^k)(w) sums, over the ways of cutting w
// into k non-empty pieces, the product of the pieces' signature coefficients.  With Q_k[j] = sum over cuts of w[0:j]
// into k pieces:  Q_1[j] = S(w[0:j]),  Q_k[j] = sum_m Q_{k-1}[m] S(w[m:j]),  logsig(w) = sum_k (-1)^{k+1} Q_k[n] / k.
constexpr int kMaxLogDepth = 12;

// DEPTH > 0: compile-time bound on the word length, all loops unrolled so that the small tables stay in registers;
// DEPTH == 0: any length up to kMaxLogDepth (tables in scratch memory).
template <int DEPTH>
__global__ void logsig_forward_kernel(const float* __restrict__ coeffs, int64_t B, int64_t nW, const int32_t* __restrict__ lyn_len,
                                      const int32_t* __restrict__ lyn_sub, int64_t n_lyn, int stride, int depth,
                                      float* __restrict__ out)
{
    constexpr int MD = DEPTH ? DEPTH : kMaxLogDepth;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * n_lyn) return;
    const int64_t b = idx / n_lyn, k = idx - b * n_lyn;
    const int n = lyn_len[k];
    const int32_t* sub = lyn_sub + k * stride;
    const float* S = coeffs + b * nW;
    // sw[i][j] = S(w[i:j]) for 0 <= i < j <= n
    float sw[MD][MD + 1];
#pragma unroll
    for (int i = 0; i < MD; ++i)
#pragma unroll
        for (int j = 0; j <= MD; ++j) sw[i][j] = (i < j && j <= n) ? S[sub[i * (depth + 1) + j]] : 0.0f;
    float Q[MD + 1], Qn[MD + 1];
#pragma unroll
    for (int j = 0; j <= MD; ++j) Q[j] = j == 0 ? 0.0f : sw[0][j];                  // one piece: w[0:j]
    float acc = 0.0f;
#pragma unroll
    for (int j = 1; j <= MD; ++j) acc = j == n ? Q[j] : acc;
#pragma unroll
    for (int kk = 2; kk <= MD; ++kk) {
#pragma unroll
        for (int j = 0; j <= MD; ++j) {
            float v = 0.0f;
#pragma unroll
            for (int m = 1; m < MD; ++m)
                if (m >= kk - 1 && m < j) v = fmaf(Q[m], sw[m][j], v);
            Qn[j] = v;
        }
        float qn = 0.0f;
#pragma unroll
        for (int j = 0; j <= MD; ++j) { Q[j] = Qn[j]; qn = j == n ? Qn[j] : qn; }
        if (kk <= n) acc += ((kk & 1) ? 1.0f : -1.0f) / (float)kk * qn;
    }
    out[idx] = acc;
}

// d logsig(w) / d S(w[i:j]) = sum_{a, c >= 0} (-1)^{a+c} / (a + c + 1) * Pre_a[i] * Suf_c[j], with Pre_a[i] the sum over
// cuts of w[0:i] into a pieces (Pre_0[0] = 1) and Suf_c[j] the same for w[j:n] (Suf_0[n] = 1).  Sub-words are shared
// between Lyndon words (a single letter by thousands of them), so the contributions are not added with atomics:
// this kernel writes them to part[(b n_lyn + k) n_pairs + pair(i, j)] and logsig_gather_kernel sums, per sub-word,
// the entries an inverse table lists.
// emit(i, j, value) receives g * d logsig(w) / d S(w[i:j]) for every 0 <= i < j <= n
template <int MD, class Emit>
__device__ __forceinline__ void logsig_word_adjoint(const float* __restrict__ S, const int32_t* __restrict__ sub, int n, int depth,
                                                    float g, Emit&& emit)
{
    float sw[MD][MD + 1];
#pragma unroll
    for (int i = 0; i < MD; ++i)
#pragma unroll
        for (int j = 0; j <= MD; ++j) sw[i][j] = (i < j && j <= n) ? S[sub[i * (depth + 1) + j]] : 0.0f;
    // pre[a][i], suf[c][j] for a, c = 0..n-1 (pieces that reach beyond n are zero through sw)
    float pre[MD][MD + 1], suf[MD][MD + 1];
#pragma unroll
    for (int i = 0; i <= MD; ++i) { pre[0][i] = i == 0 ? 1.0f : 0.0f; suf[0][i] = i == n ? 1.0f : 0.0f; }
#pragma unroll
    for (int a = 1; a < MD; ++a)
#pragma unroll
        for (int i = 0; i <= MD; ++i) {
            float v = 0.0f, u = 0.0f;
#pragma unroll
            for (int m = 0; m < MD; ++m)
                if (m < i) v = fmaf(pre[a - 1][m], sw[m][i], v);
#pragma unroll
            for (int m = 1; m <= MD; ++m)
                if (m > i && i < MD) u = fmaf(sw[i < MD ? i : 0][m], suf[a - 1][m], u);
            pre[a][i] = v;
            suf[a][i] = u;
        }
#pragma unroll
    for (int i = 0; i < MD; ++i)
#pragma unroll
        for (int j = i + 1; j <= MD; ++j) {
            if (j > n) continue;
            float t = 0.0f;
#pragma unroll
            for (int a = 0; a < MD; ++a)
#pragma unroll
                for (int c = 0; c < MD; ++c)
                    if (a + c < MD) t = fmaf((((a + c) & 1) ? -1.0f : 1.0f) / (float)(a + c + 1), pre[a][i] * suf[c][j], t);
            emit(i, j, g * t);
        }
}

template <int DEPTH>
__global__ void logsig_backward_kernel(const float* __restrict__ coeffs, const float* __restrict__ glog, int64_t B, int64_t nW,
                                       const int32_t* __restrict__ lyn_len, const int32_t* __restrict__ lyn_sub, int64_t n_lyn,
                                       int stride, int depth, int n_pairs, float* __restrict__ part)
{
    constexpr int MD = DEPTH ? DEPTH : kMaxLogDepth;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * n_lyn) return;
    const int64_t b = idx / n_lyn, k = idx - b * n_lyn;
    float* dst = part + idx * n_pairs;
    logsig_word_adjoint<MD>(coeffs + b * nW, lyn_sub + k * stride, lyn_len[k], depth, glog[idx], [&](int i, int j, float v) {
        dst[i * depth - i * (i - 1) / 2 + (j - i - 1)] = v;                     // pairs i < j <= depth in row-major order
    });
}

// One workgroup per path, for word sets whose gradient row fits in LDS: the contributions are added there with LDS
// atomics (sub-words shared by many Lyndon words meet in one address, but only within a workgroup) and the row is
// stored once.  Neither the array of contributions nor the inverse table is needed.
template <int DEPTH>
__global__ __launch_bounds__(512) void logsig_backward_lds_kernel(const float* __restrict__ coeffs, const float* __restrict__ glog,
                                                                  int64_t nW, const int32_t* __restrict__ lyn_len,
                                                                  const int32_t* __restrict__ lyn_sub, int64_t n_lyn, int stride,
                                                                  int depth, float* __restrict__ gcoeffs)
{
    constexpr int MD = DEPTH ? DEPTH : kMaxLogDepth;
    extern __shared__ float4 logsig_smem[];
    float* const acc = (float*)logsig_smem;
    const int64_t b = blockIdx.x;
    for (int64_t u = threadIdx.x; u < nW; u += blockDim.x) acc[u] = 0.0f;
    __syncthreads();
    const float* S = coeffs + b * nW;
    for (int64_t k = threadIdx.x; k < n_lyn; k += blockDim.x) {
        const int32_t* sub = lyn_sub + k * stride;
        logsig_word_adjoint<MD>(S, sub, lyn_len[k], depth, glog[b * n_lyn + k], [&](int i, int j, float v) {
            __hip_atomic_fetch_add(acc + sub[i * (depth + 1) + j], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        });
    }
    __syncthreads();
    for (int64_t u = threadIdx.x; u < nW; u += blockDim.x) gcoeffs[b * nW + u] = acc[u];
}

// one wavefront per (path, sub-word): the lists of short sub-words are thousands of entries long
__global__ __launch_bounds__(256) void logsig_gather_kernel(const float* __restrict__ part, int64_t B, int64_t nW, int64_t n_lyn,
                                                            int n_pairs, const int32_t* __restrict__ inv_off,
                                                            const int32_t* __restrict__ inv, float* __restrict__ gcoeffs)
{
    const int lane = threadIdx.x & 63;
    const int64_t idx = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (idx >= B * nW) return;
    const int64_t b = idx / nW, u = idx - b * nW;
    const float* src = part + b * n_lyn * n_pairs;
    float acc = 0.0f;
    for (int32_t e = inv_off[u] + lane; e < inv_off[u + 1]; e += 64) acc += src[inv[e]];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) gcoeffs[idx] = acc;
}

hipError_t logsig_forward(const float* coeffs, int64_t B, int64_t nW, const int32_t* lyn_len, const int32_t* lyn_sub, int64_t n_lyn,
                          int stride, int depth, float* out, hipStream_t stream)
{
    const int64_t n = B * n_lyn;
    if (n <= 0) return hipSuccess;
    if (depth > kMaxLogDepth) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((n + 127) / 128);
#define SIG_LOGSIG_FWD(DEPTH) logsig_forward_kernel<DEPTH><<<grid, 128, 0, stream>>>(coeffs, B, nW, lyn_len, lyn_sub, n_lyn, stride, depth, out)
    if (depth <= 4) SIG_LOGSIG_FWD(4);
    else if (depth <= 6) SIG_LOGSIG_FWD(6);
    else if (depth <= 8) SIG_LOGSIG_FWD(8);
    else SIG_LOGSIG_FWD(0);
#undef SIG_LOGSIG_FWD
    return hipGetLastError();
}
// bytes of LDS the one-kernel form of the backward needs for a gradient row; 0 = the row does not fit
static size_t logsig_row_lds_bytes(int64_t nW, bool two_kernels)
{
    if (two_kernels) return 0;                                   // the tests force the two-kernel form
    const size_t n = ((size_t)nW * sizeof(float) + 15) & ~(size_t)15;
    return n <= 128 * 1024 ? n : 0;
}

hipError_t logsig_backward(const float* coeffs, const float* glog, int64_t B, int64_t nW, const int32_t* lyn_len,
                           const int32_t* lyn_sub, int64_t n_lyn, int stride, int depth, int n_pairs, const int32_t* inv_off,
                           const int32_t* inv, float* part, float* gcoeffs, bool two_kernels, hipStream_t stream)
{
    const int64_t n = B * n_lyn;
    if (B <= 0) return hipSuccess;
    if (depth > kMaxLogDepth) return hipErrorInvalidValue;
    if (const size_t lds = logsig_row_lds_bytes(nW, two_kernels)) {
        if (B > 0x7fffffff) return hipErrorInvalidValue;
#define SIG_LOGSIG_BWD_LDS(DEPTH)                                                                                              \
    do {                                                                                                                       \
        if (lds > 64 * 1024) {                                                                                                 \
            hipError_t ea = ensure_dynamic_lds(reinterpret_cast<const void*>(&logsig_backward_lds_kernel<DEPTH>), 128 * 1024); \
            if (ea != hipSuccess) return ea;                                                                                   \
        }                                                                                                                      \
        logsig_backward_lds_kernel<DEPTH><<<(unsigned)B, 512, lds, stream>>>(coeffs, glog, nW, lyn_len, lyn_sub, n_lyn, stride, \
                                                                            depth, gcoeffs);                                   \
    } while (0)
        if (depth <= 4) SIG_LOGSIG_BWD_LDS(4);
        else if (depth <= 6) SIG_LOGSIG_BWD_LDS(6);
        else if (depth <= 8) SIG_LOGSIG_BWD_LDS(8);
        else SIG_LOGSIG_BWD_LDS(0);
#undef SIG_LOGSIG_BWD_LDS
        return hipGetLastError();
    }
    if (n <= 0) {                                          // no Lyndon words: the gradient is zero
        return fill_zero(gcoeffs, B * nW, stream);
    }
    if (!part) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((n + 127) / 128);
#define SIG_LOGSIG_BWD(DEPTH) \
    logsig_backward_kernel<DEPTH><<<grid, 128, 0, stream>>>(coeffs, glog, B, nW, lyn_len, lyn_sub, n_lyn, stride, depth, n_pairs, part)
    if (depth <= 4) SIG_LOGSIG_BWD(4);
    else if (depth <= 6) SIG_LOGSIG_BWD(6);
    else if (depth <= 8) SIG_LOGSIG_BWD(8);
    else SIG_LOGSIG_BWD(0);
#undef SIG_LOGSIG_BWD
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t m = (B * nW + 3) / 4;                  // four wavefronts per workgroup
    if (m > 0x7fffffff) return hipErrorInvalidValue;
    logsig_gather_kernel<<<(unsigned)m, 256, 0, stream>>>(part, B, nW, n_lyn, n_pairs, inv_off, inv, gcoeffs);
    return hipGetLastError();
}

// Register-only multiply-add loop for the benchmark: every thread runs `iters` rounds of 16 independent fmaf chains
// (no memory traffic inside the loop) and stores one value so that nothing is optimised away.  The multiplier and the
// addend differ from lane to lane, so all three operands of every instruction are vector registers, as in the
// signature kernels (with a scalar-register operand the same loop was measured at two thirds of the rate).
__global__ __launch_bounds__(256) void fma_probe_kernel(float* out, int iters, float a, float b)
{
    float x[16];
    a += (float)threadIdx.x * 1e-7f;
    b += (float)threadIdx.x * 1e-8f;
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = (float)(threadIdx.x + i);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = fmaf(x[i], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Issue-rate probes (register-only loops; per iteration 64 vector multiply-adds and / or 8 matrix instructions):
//   MODE 0  64 v_fma_f32 whose three operands are vector registers
//   MODE 1  64 v_fma_f32 with the multiplier in a scalar register (lane-uniform kernel argument)
//   MODE 2  8 v_mfma_f32_16x16x4_f32 (independent accumulators)
//   MODE 3  the 64 multiply-adds of MODE 0 interleaved with the 8 matrix instructions of MODE 2
// Timed with one and with several wavefronts per SIMD they show what a lone wavefront can issue, whether vector and
// matrix instructions overlap, and what a scalar operand costs.
typedef float probe_v4f __attribute__((ext_vector_type(4)));
template <int MODE>
__global__ __launch_bounds__(256) void issue_probe_kernel(float* out, int iters, float a0, float b0)
{
    constexpr bool kVec = MODE != 2, kMat = MODE >= 2;
    float x[64];
    probe_v4f acc[8];
#pragma unroll
    for (int i = 0; i < 64; ++i) x[i] = (float)threadIdx.x * 1e-3f + (float)i;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (probe_v4f){0.0f, 0.0f, 0.0f, 0.0f};
    float a = a0, b = b0 + (float)threadIdx.x * 1e-8f;
    if (MODE != 1) a += (float)threadIdx.x * 1e-7f;      // MODE 1 keeps the multiplier lane-uniform
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (kMat) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
            if (kVec) {
#pragma unroll
                for (int j = 0; j < 8; ++j) x[8 * i + j] = fmaf(x[8 * i + j], a, b);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 64; ++i) s += x[i];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Modes 4 and 5: the same 64 multiply-adds per iteration with the registers named in the instruction, so that the
// three source operands of every instruction lie in one register bank (register number mod 4; mode 4) or in three
// different banks (mode 5).  Compiled code cannot choose: its operands fall into banks as the allocator places them.
#define SIG_PROBE_CLOBBERS "v32", "v36", "v40", "v44", "v48", "v52", "v56", "v60", "v64", "v65", "v68", "v69", "v70"
#define SIG_PROBE_ROUND(M, A)                                                                                          \
    "v_fma_f32 v32, v32, " M ", " A "\n v_fma_f32 v36, v36, " M ", " A "\n v_fma_f32 v40, v40, " M ", " A "\n"           \
    "v_fma_f32 v44, v44, " M ", " A "\n v_fma_f32 v48, v48, " M ", " A "\n v_fma_f32 v52, v52, " M ", " A "\n"           \
    "v_fma_f32 v56, v56, " M ", " A "\n v_fma_f32 v60, v60, " M ", " A "\n"
#define SIG_PROBE_BODY(M, A)                                                                                           \
    SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A)                           \
    SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A) SIG_PROBE_ROUND(M, A)
// VARIANT 0: all three sources in bank 0; 1: three banks; 2: accumulator and multiplier share bank 0, addend in bank 2;
// 3: multiplier and addend share bank 1, accumulator in bank 0
template <int VARIANT>
__global__ __launch_bounds__(256) void bank_probe_kernel(float* out, int iters)
{
    // accumulators 1.0, multipliers 0.999, addends 0.001 (v64 / v68: bank 0 like the accumulators; v65 / v69: bank 1; v70: bank 2)
    asm volatile("v_mov_b32 v32, 1.0\n v_mov_b32 v36, 1.0\n v_mov_b32 v40, 1.0\n v_mov_b32 v44, 1.0\n"
                 "v_mov_b32 v48, 1.0\n v_mov_b32 v52, 1.0\n v_mov_b32 v56, 1.0\n v_mov_b32 v60, 1.0\n"
                 "v_mov_b32 v64, 0x3f7fbe77\n v_mov_b32 v65, 0x3f7fbe77\n v_mov_b32 v68, 0x3a83126f\n v_mov_b32 v70, 0x3a83126f\n"
                 "v_mov_b32 v69, 0x3a83126f\n"
                 ::: SIG_PROBE_CLOBBERS);
    for (int it = 0; it < iters; ++it) {
        if (VARIANT == 0) asm volatile(SIG_PROBE_BODY("v64", "v68") ::: SIG_PROBE_CLOBBERS);
        else if (VARIANT == 1) asm volatile(SIG_PROBE_BODY("v65", "v70") ::: SIG_PROBE_CLOBBERS);
        else if (VARIANT == 2) asm volatile(SIG_PROBE_BODY("v64", "v70") ::: SIG_PROBE_CLOBBERS);
        else asm volatile(SIG_PROBE_BODY("v65", "v69") ::: SIG_PROBE_CLOBBERS);
    }
    float s;
    asm volatile("v_add_f32 %0, v32, v60\n" : "=v"(s) :: SIG_PROBE_CLOBBERS);
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

hipError_t issue_probe(float* out, int blocks, int iters, int mode, hipStream_t stream)
{
    if (blocks <= 0 || iters <= 0 || mode < 0 || mode > 7) return hipErrorInvalidValue;
    if (mode == 4) bank_probe_kernel<0><<<(unsigned)blocks, 256, 0, stream>>>(out, iters);
    if (mode == 5) bank_probe_kernel<1><<<(unsigned)blocks, 256, 0, stream>>>(out, iters);
    if (mode == 6) bank_probe_kernel<2><<<(unsigned)blocks, 256, 0, stream>>>(out, iters);
    if (mode == 7) bank_probe_kernel<3><<<(unsigned)blocks, 256, 0, stream>>>(out, iters);
    if (mode >= 4) return hipGetLastError();
    switch (mode) {
        case 0: issue_probe_kernel<0><<<(unsigned)blocks, 256, 0, stream>>>(out, iters, 0.999f, 0.001f); break;
        case 1: issue_probe_kernel<1><<<(unsigned)blocks, 256, 0, stream>>>(out, iters, 0.999f, 0.001f); break;
        case 2: issue_probe_kernel<2><<<(unsigned)blocks, 256, 0, stream>>>(out, iters, 0.999f, 0.001f); break;
        default: issue_probe_kernel<3><<<(unsigned)blocks, 256, 0, stream>>>(out, iters, 0.999f, 0.001f); break;
    }
    return hipGetLastError();
}

hipError_t fma_probe(float* out, int blocks, int iters, hipStream_t stream)
{
    if (blocks <= 0 || iters <= 0) return hipErrorInvalidValue;
    fma_probe_kernel<<<(unsigned)blocks, 256, 0, stream>>>(out, iters, 0.999f, 0.001f);
    return hipGetLastError();
}

hipError_t fill_zero(float* p, int64_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    const int threads = 256;
    fill_zero_kernel<<<(unsigned)((n + threads - 1) / threads), threads, 0, stream>>>(p, n);
    return hipGetLastError();
}

hipError_t grad_points(const float* gdx, int64_t B, int64_t P, int d, float* grad_path, hipStream_t stream)
{
    const int64_t n = B * P * d;
    if (n <= 0) return hipSuccess;
    const int threads = 256;
    grad_points_kernel<<<(unsigned)((n + threads - 1) / threads), threads, 0, stream>>>(gdx, B, P, d, grad_path);
    return hipGetLastError();
}

hipError_t static_scratch(void** ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex m;
    static void* per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(m);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // this device's copy of the array
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255) != 0) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

}  // namespace sig
