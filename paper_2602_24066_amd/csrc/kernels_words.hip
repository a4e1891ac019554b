// Time chunks for word sets that are closed under prefixes and suffixes (every anisotropic set, Definition 7.1; word
// lists that happen to be): Chen's relation (eq. 2) restricted to such a set needs nothing outside it,
//   (a (x) b)(w) = a(w) + b(w) + sum_{m=1..n-1} a(w_1..w_m) b(w_{m+1}..w_n)        (product of Section 2.1),
// so the signatures of the C chunks of a path, computed side by side as independent rows, are multiplied afterwards,
// and the backward pass of chunk c starts from the product of the first c + 1 chunk signatures and from the adjoint
//   Abar_c(u) = grad(u) + sum_{v: u v in W} grad(u v) Q_c(v),   Q_c = S_{c+1} (x) .. (x) S_{C-1}
// (Proposition 4.1 with the right factor taken at a chunk boundary).  Both sums run over the same terms (w, m); the
// host lists them once per order of use, two 16-bit word indices per entry: by word w for the product, by prefix
// u = w_1..w_m (with u beside every term) for the adjoint.  The signatures lie in LDS (one path per workgroup), the
// tables stream from L2.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.hpp"

namespace sig {
namespace {

constexpr int kWordsThreads = 1024;      // sixteen wavefronts: the gathers are latency-bound

// The terms of one word of the product: their table entries are fetched for two words before either is used (the
// entries come from L2, the factors from LDS).
struct WordTerms {
    uint32_t pr[8];
    const uint32_t* pp;
    int cnt, n;
};
__device__ __forceinline__ void fetch_terms(const WordTables& t, int w, int& n, WordTerms& x)
{
    while (w >= t.level_start[n + 1]) ++n;                            // length of w: grows with w
    x.n = n;
    x.cnt = t.level_start[n + 1] - t.level_start[n];
    x.pp = t.prod_pairs + t.tail_off[n] + (w - t.level_start[n]);
#pragma unroll
    for (int m = 0; m < 8; ++m) x.pr[m] = m < n - 1 ? x.pp[(size_t)m * x.cnt] : 0u;
}
__device__ __forceinline__ float sum_terms(const WordTerms& x, const float* a, const float* b, float acc)
{
#pragma unroll
    for (int m = 0; m < 8; ++m)
        if (m < x.n - 1) acc = fmaf(a[x.pr[m] & 0xffffu], b[x.pr[m] >> 16], acc);
    for (int m = 8; m < x.n - 1; ++m) {
        const uint32_t pr = x.pp[(size_t)m * x.cnt];
        acc = fmaf(a[pr & 0xffffu], b[pr >> 16], acc);
    }
    return acc;
}

// out = a (x) b on the word set; a, b, out: LDS rows of t.W floats (out distinct from a and b)
__device__ __forceinline__ void words_product(const WordTables& t, const float* a, const float* b, float* out, int tid)
{
    int n0 = 1, n1 = 1;
    for (int w0 = tid; w0 < t.W; w0 += 2 * kWordsThreads) {
        const int w1 = w0 + kWordsThreads;
        WordTerms x0, x1;
        fetch_terms(t, w0, n0, x0);
        if (w1 < t.W) fetch_terms(t, w1, n1, x1);
        out[w0] = sum_terms(x0, a, b, a[w0] + b[w0]);
        if (w1 < t.W) out[w1] = sum_terms(x1, a, b, a[w1] + b[w1]);
    }
}

__device__ __forceinline__ void copy_row(const float* src, float* dst, int n, int tid)
{
    for (int i = tid; i < n; i += kWordsThreads) dst[i] = src[i];
}

// One workgroup per path.  S: chunk signatures [B][C][W].  Forward scan (reverse = 0): P_c = S_0 (x) .. (x) S_c, the
// signature at the end of chunk c, to row c of `rows` [B][C][W] if given; the last product also to `last` [B][W] if
// given.  Reverse scan: Q_c = S_{c+1} (x) .. (x) S_{C-1} for c = C-2 .. 0 to row c of `rows` (row C-1 is not written).
__global__ __launch_bounds__(kWordsThreads) void words_scan_kernel(WordTables t, const float* __restrict__ S, int C, int reverse,
                                                                   float* __restrict__ rows, float* __restrict__ last,
                                                                   float* __restrict__ rows_reverse)
{
    extern __shared__ float sm[];
    const int tid = threadIdx.x;
    // both scans in one launch: the second layer of workgroups runs the reverse scan into rows_reverse
    if (blockIdx.y == 1) {
        reverse = 1;
        rows = rows_reverse;
        last = nullptr;
    }
    const int64_t b = blockIdx.x;
    const int W = t.W;
    float* acc = sm;
    float* nxt = sm + W;
    float* out = sm + 2 * W;
    const float* Sb = S + b * (int64_t)C * W;
    float* Rb = rows ? rows + b * (int64_t)C * W : nullptr;
    if (!reverse) {
        copy_row(Sb, acc, W, tid);
        copy_row(Sb + W, nxt, W, tid);
        __syncthreads();
        if (Rb) copy_row(acc, Rb, W, tid);
        for (int c = 1; c < C; ++c) {
            words_product(t, acc, nxt, out, tid);
            __syncthreads();
            if (c + 1 < C) copy_row(Sb + (int64_t)(c + 1) * W, nxt, W, tid);   // nxt was read before the barrier
            if (Rb) copy_row(out, Rb + (int64_t)c * W, W, tid);
            if (c == C - 1 && last) copy_row(out, last + b * (int64_t)W, W, tid);
            float* sw = acc; acc = out; out = sw;
            __syncthreads();
        }
    } else {
        copy_row(Sb + (int64_t)(C - 1) * W, acc, W, tid);
        if (C > 2) copy_row(Sb + (int64_t)(C - 2) * W, nxt, W, tid);
        __syncthreads();
        if (Rb) copy_row(acc, Rb + (int64_t)(C - 2) * W, W, tid);
        for (int c = C - 2; c >= 1; --c) {
            words_product(t, nxt, acc, out, tid);                               // S_c (x) Q_c
            __syncthreads();
            if (c - 1 >= 1) copy_row(Sb + (int64_t)(c - 1) * W, nxt, W, tid);
            if (Rb) copy_row(out, Rb + (int64_t)(c - 1) * W, W, tid);
            float* sw = acc; acc = out; out = sw;
            __syncthreads();
        }
    }
}

// One step of an inclusive sum within runs of equal keys: the lane the pattern names as source adds its value where it
// carries the same key; lanes the pattern gives no source keep theirs (their source key reads as 0xffffffff, no word).
template <int CTRL, int ROWS>
__device__ __forceinline__ void seg_step(float& v, uint32_t key)
{
    const uint32_t ks = (uint32_t)__builtin_amdgcn_update_dpp((int)0xffffffffu, (int)key, CTRL, ROWS, 0xf, false);
    const float vs = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xf, false));
    if (ks == key) v += vs;
}

// One workgroup per (path, chunk but the last).  grad [B][W], Q [B][C][W] (row c: what follows chunk c), Abar [B][C][W]
// (rows of last chunks are left alone: their adjoint is the gradient itself).  The gradient row and Q are staged in LDS before anything is written, so
// Abar may be the array Q itself.  The terms lie sorted by their prefix u: a wavefront takes 64 consecutive terms (four
// such groups in flight), sums runs of equal u within each row of 16 lanes and adds every run's sum to u's accumulator
// in LDS.
__global__ __launch_bounds__(kWordsThreads) void words_adjoint_kernel(WordTables t, const float* __restrict__ grad, const float* Q,
                                                                      int C, float* Abar, float* __restrict__ zeroed, int64_t n_zeroed)
{
    // an array the caller wants cleared on the way (the gradient of the path, which the chain rule adds into): every
    // workgroup clears its share
    if (zeroed) {
        const int64_t per = (n_zeroed + gridDim.x - 1) / gridDim.x, lo = per * blockIdx.x;
        const int64_t hi = lo + per < n_zeroed ? lo + per : n_zeroed;
        for (int64_t i = lo + threadIdx.x; i < hi; i += kWordsThreads) zeroed[i] = 0.0f;
    }
    extern __shared__ float sm[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NWAVES = kWordsThreads / 64, UN = 4;
    const int64_t b = blockIdx.x / (C - 1);
    const int64_t row = b * C + (blockIdx.x - b * (C - 1));             // b * C + c, c < C - 1
    const int W = t.W;
    float* out = Abar + row * (int64_t)W;
    float* g = sm;
    float* q = sm + W;
    float* acc = sm + 2 * W;                                            // [W + 1]: the last entry takes the padding
    for (int i = tid; i < W; i += kWordsThreads) {
        const float v = grad[b * (int64_t)W + i];
        g[i] = v;
        acc[i] = v;
        q[i] = Q[row * (int64_t)W + i];
    }
    if (tid == 0) acc[W] = 0.0f;
    __syncthreads();
    for (int grp = wave; grp < t.adj_groups; grp += NWAVES) {
        uint32_t pr[UN], key[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            pr[j] = t.adj_pairs[(size_t)grp * 256 + j * 64 + lane];
            key[j] = t.adj_key[(size_t)grp * 256 + j * 64 + lane];
        }
        float v[UN];
#pragma unroll
        for (int j = 0; j < UN; ++j) v[j] = g[pr[j] & 0xffffu] * q[pr[j] >> 16];
        // inclusive sums within runs of equal keys, per row of 16 lanes (keys ascend along the lanes, so equal ends mean
        // an equal run)
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            seg_step<0x111, 0xf>(v[j], key[j]);     // row_shr:1
            seg_step<0x112, 0xf>(v[j], key[j]);     // row_shr:2
            seg_step<0x114, 0xf>(v[j], key[j]);     // row_shr:4
            seg_step<0x118, 0xf>(v[j], key[j]);     // row_shr:8
        }
#pragma unroll
        for (int j = 0; j < UN; ++j) {
            // the last lane of a run within its row holds the run's sum there: the next lane's key differs (row_shl:1; a
            // row's last lane always adds)
            const uint32_t kd = (uint32_t)__builtin_amdgcn_update_dpp((int)0xffffffffu, (int)key[j], 0x101, 0xf, 0xf, false);
            if (kd != key[j]) atomicAdd(&acc[key[j]], v[j]);
        }
    }
    __syncthreads();
    for (int i = tid; i < W; i += kWordsThreads) out[i] = acc[i];
}

}  // namespace

size_t words_scan_lds_bytes(int64_t W) { return 3 * (size_t)W * sizeof(float); }

hipError_t words_scan(const WordTables& t, const float* S, int64_t B, int C, bool reverse, float* rows, float* last,
                      hipStream_t stream)
{
    if (B < 1 || C < 2 || B > 0x7fffffff || t.W < 1 || t.W > 0xffff) return hipErrorInvalidValue;
    const size_t lds = words_scan_lds_bytes(t.W);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&words_scan_kernel), (int)(160 * 1024));
        if (e != hipSuccess) return e;
    }
    words_scan_kernel<<<(unsigned)B, kWordsThreads, lds, stream>>>(t, S, C, reverse ? 1 : 0, rows, last, nullptr);
    return hipGetLastError();
}

hipError_t words_scan_both(const WordTables& t, const float* S, int64_t B, int C, float* rows_forward, float* rows_reverse,
                           hipStream_t stream)
{
    if (B < 1 || C < 2 || B > 0x7fffffff || t.W < 1 || t.W > 0xffff || !rows_forward || !rows_reverse) return hipErrorInvalidValue;
    const size_t lds = words_scan_lds_bytes(t.W);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&words_scan_kernel), (int)(160 * 1024));
        if (e != hipSuccess) return e;
    }
    words_scan_kernel<<<dim3((unsigned)B, 2), kWordsThreads, lds, stream>>>(t, S, C, 0, rows_forward, nullptr, rows_reverse);
    return hipGetLastError();
}

hipError_t words_adjoint(const WordTables& t, const float* grad, const float* Q, int64_t B, int C, float* Abar, float* zeroed,
                         int64_t n_zeroed, hipStream_t stream)
{
    if (B < 1 || C < 2 || B * (C - 1) > 0x7fffffff || t.W < 1 || t.W > 0xffff) return hipErrorInvalidValue;
    const size_t lds = (3 * (size_t)t.W + 1) * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&words_adjoint_kernel), (int)(160 * 1024));
        if (e != hipSuccess) return e;
    }
    words_adjoint_kernel<<<(unsigned)(B * (C - 1)), kWordsThreads, lds, stream>>>(t, grad, Q, C, Abar, zeroed, n_zeroed);
    return hipGetLastError();
}

}  // namespace sig
