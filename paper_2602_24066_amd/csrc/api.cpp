// C ABI of the library (see include/sig.h for the contract of every entry point).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include <cstdlib>
#include <mutex>
#include <string>

#include "../../include/sig.h"
#include "jit.hpp"
#include "kernels.hpp"
#include "wordset.hpp"

struct sig_wordset : public sig::WordSet {};

namespace {
thread_local int g_last_hip = 0;

int hip_fail(hipError_t e)
{
    g_last_hip = (int)e;
    return SIG_EHIP;
}

const sig::WordSet* W(const sig_wordset* ws) { return ws; }

// Launch-shape knobs: one table for the environment variables read when a set is built and for
// sig_wordset_set_option / sig_wordset_get_option.
struct OptionName { const char* name; const char* env; int sig::WordSet::Options::*field; };
const OptionName kOptions[] = {
    {"no_jit", "SIG_NO_JIT", &sig::WordSet::Options::no_jit},
    {"jit_waves", "SIG_JIT_WAVES", &sig::WordSet::Options::jit_waves},
    {"chunks", "SIG_CHUNKS", &sig::WordSet::Options::chunks},
    {"fwd_tails", "SIG_FWD_TAILS", &sig::WordSet::Options::fwd_tails},
    {"bwd_tails", "SIG_BWD_TAILS", &sig::WordSet::Options::bwd_tails},
    {"lanes", "SIG_LANES", &sig::WordSet::Options::lanes},
    {"lanes_levels", "SIG_LANES_LEVELS", &sig::WordSet::Options::lanes_levels},
    {"logsig_gather", "SIG_LOGSIG_GATHER", &sig::WordSet::Options::logsig_gather},
    {"jit_wg_waves", "SIG_JIT_WG_WAVES", &sig::WordSet::Options::jit_wg_waves},
    {"bwd_tile", "SIG_BWD_TILE", &sig::WordSet::Options::bwd_tile},
    {"ckpt_chunks", "SIG_CKPT_CHUNKS", &sig::WordSet::Options::ckpt_chunks},
    {"jit_fwd_tile", "SIG_JIT_FWD_TILE", &sig::WordSet::Options::jit_fwd_tile},
};
void options_from_environment(sig::WordSet& w)
{
    for (const OptionName& o : kOptions) {
        const char* e = std::getenv(o.env);
        if (e && e[0]) w.opt.*(o.field) = std::atoi(e);
    }
}
int finish_build(int rc, sig::WordSet* w, sig_wordset** out)
{
    if (rc != SIG_OK) return rc;
    options_from_environment(*w);
    *out = static_cast<sig_wordset*>(w);
    return SIG_OK;
}

// Picks the plan variant: the coarsest one (least recomputation of shared ancestors) that still
// yields enough wavefronts to occupy the 256 compute units, else the finest.
int pick_variant(const sig::WordSet& ws, int dir, int64_t B, int64_t want = 2048 /* two wavefronts per SIMD */)
{
    const int64_t groups = (B + 63) / 64;
    const auto& pl = ws.plans[dir];
    for (size_t v = 0; v < pl.size(); ++v)
        if ((int64_t)pl[v].units.size() * groups >= want) return (int)v;
    return (int)pl.size() - 1;
}

// kernel timer (see sig_profile_enable); channels 0/1: main kernel of forward/backward, 2/3: whole call
struct Profiler {
    unsigned mask = 0;                // bit `which` set: that channel records
    std::vector<hipEvent_t> ev[4];    // start/stop interleaved
    size_t used[4] = {0, 0, 0, 0};
    hipEvent_t* next(int dir)
    {
        if (!((mask >> dir) & 1u) || used[dir] >= SIG_PROFILE_MAX_LAUNCHES) return nullptr;
        if (ev[dir].size() < 2 * (used[dir] + 1)) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return nullptr;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return nullptr; }
            ev[dir].push_back(a);
            ev[dir].push_back(b);
        }
        return &ev[dir][2 * used[dir]++];
    }
};
Profiler g_prof;

// brackets everything a call enqueues
struct CallTimer {
    hipEvent_t* pe;
    hipStream_t st;
    CallTimer(int dir, hipStream_t s) : pe(g_prof.next(2 + dir)), st(s) { if (pe) (void)hipEventRecord(pe[0], st); }
    ~CallTimer() { if (pe) (void)hipEventRecord(pe[1], st); }
};

// Time chunks for full truncations: with few paths the sequential kernels leave wavefront slots empty, so the
// segments of every path are cut into C chunks that run as independent rows and are combined afterwards with Chen's
// relation.  Measured on the three instantiated shapes this pays off for the forward kernels once a chunk is a
// few hundred segments long (the chunk products and the second launch cost about as much as 100 segments); a
// chunked backward pass that starts from the terminal signature alone has to recompute the chunk signatures, a forward
// pass of its own, so sig_backward chunks on request (option "chunks") and, by itself, only where four or more chunks
// fit (few long paths, see below); otherwise the checkpointed calls, which keep the chunk signatures, are the way to
// more rows.
struct Chunks { int64_t C, Lc; };
// own_chunks = false: sig_backward does not chunk by itself (sig_backward_static, whose scratch array is sized for
// whole paths).
Chunks trunc_chunks(const sig::WordSet& w, int dir, int64_t B, int64_t n_points, bool own_chunks = true)
{
    const int64_t L = n_points - 1;
    int64_t C = 1;
    if (L >= 64 && sig::chunking_available(w.d, w.depth)) {
        if (w.opt.chunks > 0) {                                                           // tuning knob
            C = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(w.opt.chunks, 64), L / 32));
        } else if (dir == 0) {
            const int64_t slots = (int64_t)1024 * sig::trunc_occupancy(w.d, w.depth, dir);
            C = slots / sig::trunc_waves_per_row(w.d, w.depth, dir) / std::max<int64_t>(B, 1);
            C = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(C, 64), L / 256));
        } else if (own_chunks && !sig::trunc_backward_tails_available(w.d, w.depth)) {
            // few long paths: even with the chunk signatures recomputed, four to sixteen chunks side by side beat a walk
            // over whole paths that leaves most SIMDs empty (measured, d = 16: 8 paths x 8,192 segments 3.92 -> 1.00 ms,
            // 32 x 4,096 2.00 -> 1.09 ms; d = 8: 16 x 4,096 2.63 -> 0.67 ms, 64 x 2,048 1.33 -> 0.74 ms); with two
            // chunks the second forward pass eats the gain
            const int64_t rows_wanted = 2048 / sig::trunc_waves_per_row(w.d, w.depth, 1);
            C = std::min<int64_t>(std::min<int64_t>(16, rows_wanted / std::max<int64_t>(B, 1)), L / 256);
            C = C >= 16 ? 16 : (C >= 8 ? 8 : (C >= 4 ? 4 : 1));     // whole wavefronts per SIMD: 12 chunks lost to 8 when measured
        }
    }
    const int64_t Lc = (L + C - 1) / C;
    return Chunks{(L + Lc - 1) / Lc, Lc};
}
// Forward for d = 4 in the layout with 64 words of length 3 per wavefront (two wavefronts per chunk of a path, 2 or 4
// chunks per path in one workgroup, chunk signatures multiplied in LDS).  Returns the number of chunks, 0 = the
// kernel with four wavefronts per path instead (with its chunk arrays in HBM for long paths): measured faster only
// for fewer than 192 paths of more than 512 segments.  Four chunks need a compute unit per path, so larger batches
// take two.  The option "fwd_tails" = 0 (or a "chunks" setting) switches it off, = 2 / = 4 force that many chunks.
int64_t trunc_forward_fused_chunks(const sig::WordSet& w, int64_t B, int64_t n_points, const float* coeffs)
{
    if (!sig::trunc_forward_tails_available(w.d, w.depth) || ((uintptr_t)coeffs & 15) != 0) return 0;
    const int64_t L = n_points - 1;
    const int f = w.opt.fwd_tails;
    if (f == 0) return 0;
    if (f == -1 && w.opt.chunks > 0) return 0;               // asks for the form with chunk arrays in HBM
    int64_t C;
    if (f == 2 || f == 4) {
        C = f;
    } else {
        if (B < 192 && L > 512) return 0;
        C = B <= 256 ? 4 : 2;
    }
    while (C > 1 && L < 8 * C) C /= 2;                       // chunks of at least 8 segments
    if (C < 2) return 0;
    const int64_t Lc = (L + C - 1) / C;
    return (C - 1) * Lc >= L ? 0 : C;
}

// Backward launch shape for a full truncation.  d = 4 has a second kernel with one wavefront per (path, chunk) row
// that does half the vector work per path and fits two wavefronts on a SIMD, so it wants about two thousand rows.
// Smaller batches take its fused form (2, 4 or 8 chunks of a path in one workgroup, everything between the chunks
// in LDS), larger ones run it unchunked; the thresholds come from a scan over 64..2,048 paths of 64..1,024 segments.
// The option "bwd_tails" = 0 switches it off, = 1 takes the unfused form with chunk arrays in HBM ("chunks" chunks),
// =2 / =4 / =8 force the fused form with that many chunks.
struct BwdShape { bool tails, fused; int64_t C, Lc; };
BwdShape trunc_backward_shape(const sig::WordSet& w, int64_t B, int64_t n_points, bool own_chunks = true)
{
    const int64_t L = n_points - 1;
    const Chunks ch = trunc_chunks(w, 1, B, n_points, own_chunks);
    BwdShape s{false, false, ch.C, ch.Lc};
    if (!sig::trunc_backward_tails_available(w.d, w.depth)) return s;
    const int f = w.opt.bwd_tails;
    if (f == 0) return s;
    if (f == 1) return BwdShape{true, false, ch.C, ch.Lc};
    int64_t C = f == 2 || f == 4 || f == 8 ? f : (B <= 256 ? 8 : (B <= 896 ? 4 : (B <= 1536 ? 2 : 1)));
    while (C > 1 && L < 8 * C) C /= 2;                       // chunks of at least 8 segments
    if (C == 1) return BwdShape{true, false, f == -1 ? 1 : ch.C, f == -1 ? L : ch.Lc};
    const int64_t Lc = (L + C - 1) / C;
    if ((C - 1) * Lc >= L) return s;
    return BwdShape{true, true, C, Lc};
}
// Checkpointed form (sig_forward_checkpointed / sig_backward_checkpointed): the forward pass leaves the signatures of C
// time chunks of every path in a buffer the caller keeps, and the backward pass walks the C chunks side by side
// without recomputing them.  Taken where the backward kernel of a full truncation has too few rows to put two
// wavefronts on every SIMD (eight wavefronts per row for d = 8, sixteen for d = 16); C = 2 .. 16, chunks of at least 64
// segments (measured: 8 paths x 8,192 segments, d = 16: step 4.1 ms plain, 1.43 ms with four chunks, 1.00 ms with eight).
// "ckpt_chunks" forces a count (0: this rule, 1: off).
//
// Word sets closed under suffixes as well as prefixes (anisotropic sets, Definition 7.1) that run through the
// straight-line specialised kernels (lane = row) take the same form: Chen's relation restricted to such a set stays
// inside it.  Those kernels gain from rows up to about 2,048 (32 lane groups: fewer, larger units, so less
// recomputation of shared ancestors per group), but every chunk boundary costs a product and an adjoint sum over the
// set, gathers that run at a fraction of the rate of the kernels.  Measured on 5,754 words for 64 .. 1,024 paths of
// 512 .. 4,096 segments (step time against the plain calls: -75 % for 64 paths x 4,096 segments with eight chunks,
// -35 % for 512 x 2,048 with four, -20 % for 512 x 512 with two, -5 % for 1,024 x 512 with two); more than 2,048 rows
// lose.  "ckpt_chunks" forces a count of up to 16 (chunks of at least 64 segments).
bool jit_enabled(const sig::WordSet& w);
bool words_time_chunks(const sig::WordSet& w)
{
    return w.kind != 0 && w.pair_tables && jit_enabled(w) && w.max_len <= 14 && sig::words_scan_lds_bytes(w.size()) <= 160 * 1024;
}
Chunks checkpoint_chunks(const sig::WordSet& w, int64_t B, int64_t n_points)
{
    const int64_t L = n_points - 1;
    int64_t C = 1;
    if (B >= 1 && words_time_chunks(w)) {
        if (w.opt.ckpt_chunks > 0) {
            C = std::min<int64_t>(std::min<int64_t>(w.opt.ckpt_chunks, 16), L / 64);
        } else {
            // at most 2,048 rows and chunks of at least 256 segments; batches that stay at 512 rows or below take chunks
            // down to 128 segments; never more than eight
            C = std::min<int64_t>(2048 / B, L / 256);
            if (B * std::max<int64_t>(C, 1) <= 512) C = std::min<int64_t>(2048 / B, L / 128);
            C = std::min<int64_t>(C, 8);
        }
        C = std::max<int64_t>(1, C);
        if (B * C > (int64_t)65535 * 64) C = 1;
    }
    if (w.kind == 0 && B >= 1 && B <= 65535 && sig::trunc_backward_available(w.d, w.depth) && sig::chunking_available(w.d, w.depth) &&
        !sig::trunc_backward_tails_available(w.d, w.depth)) {
        if (w.opt.ckpt_chunks > 0) {
            C = std::min<int64_t>(w.opt.ckpt_chunks, 16);
        } else {
            const int64_t rows_wanted = 2048 / sig::trunc_waves_per_row(w.d, w.depth, 1);
            C = std::min<int64_t>(std::min<int64_t>(16, (rows_wanted + B - 1) / B), L / 64);
            if (C > 4) C = C >= 16 ? 16 : (C >= 8 ? 8 : 4);         // beyond four: powers of two (whole wavefronts per SIMD)
        }
        C = std::max<int64_t>(1, std::min<int64_t>(C, L / 64));
    }
    if (C < 2) return Chunks{1, L};
    const int64_t Lc = (L + C - 1) / C;
    return Chunks{(L + Lc - 1) / Lc, Lc};
}
size_t chunk_array_bytes(const sig::WordSet& w, int64_t B, int64_t C)
{
    return ((size_t)B * (size_t)C * (size_t)w.size() * sizeof(float) + 255) & ~(size_t)255;
}

// arrays [B][C][|W|] a chunked forward pass takes from its workspace: the chunk signatures, and the partial products
// when four or more large signatures are multiplied pair by pair (two or three, and signatures that fit LDS, are
// multiplied in one kernel)
size_t forward_chunk_arrays(const sig::WordSet& w, int64_t C) { return (C >= 4 && w.size() > 8192) ? 2 : 1; }

bool use_trunc_forward(const sig::WordSet& w, int64_t B)
{
    return w.kind == 0 && B <= 65535 && sig::trunc_forward_available(w.d, w.depth);
}

bool use_trunc_backward(const sig::WordSet& w, int64_t B)
{
    return w.kind == 0 && B <= 65535 && sig::trunc_backward_available(w.d, w.depth);
}

// ---- run-time specialised kernels ------------------------------------------------------------------------
std::mutex g_jit_mutex;

// Work units asked of the balanced planner for a batch of B paths: one or two wavefronts per SIMD (1,024 on the
// chip) over the path groups, a whole number of workgroups, and not so many that units shrink to a handful of words
// (every unit recomputes the ancestors of its first word).
int jit_wg_waves(const sig::WordSet& w)   // wavefronts (units) per workgroup
{
    return w.opt.jit_wg_waves == 8 ? 8 : std::max(1, std::min(4, w.opt.jit_wg_waves));
}
int64_t jit_units(const sig::WordSet& w, int /*dir*/, int64_t B)
{
    const int kJitWaves = jit_wg_waves(w);
    int64_t want = 2048;               // two wavefronts per SIMD
    if (w.opt.jit_waves > 0) want = w.opt.jit_waves;                                       // tuning knob
    const int64_t groups = (B + 63) / 64;
    int64_t n = std::max<int64_t>(1, want / groups);
    n = std::min(n, std::max<int64_t>(1, w.size() / 8));
    return (n + kJitWaves - 1) / kJitWaves * kJitWaves;
}

// segments per LDS tile; backward also keeps one gradient tile [T][d][65] per wavefront of the workgroup (four as a
// rule) in the 64 KB of static LDS
int jit_tile_steps(int d, int dir, int nw = 4) { return std::min(8, (dir ? 192 / std::max(nw, 4) : 240) / std::max(d, 1)); }
int jit_tile_for(const sig::WordSet& w, int dir)
{
    if (dir == 0 && w.opt.jit_fwd_tile > 0) return std::max(1, std::min(std::min(w.opt.jit_fwd_tile, 32), 240 / std::max(w.d, 1)));
    return std::max(1, jit_tile_steps(w.d, dir, jit_wg_waves(w)));
}

bool jit_enabled(const sig::WordSet& w)
{
    if (w.opt.no_jit) return false;
    return w.kernels_supported && w.size() > 0 && jit_tile_steps(w.d, 1) >= 1;
}

// The balanced plan (and kernel slot) for (direction, batch size); created on first use.  Registers bound the unit
// size: a forward unit keeps one value per word, a backward unit two, next to the Horner intermediates.
sig::WordSet::JitEntry* jit_entry(const sig::WordSet& cw, int dir, int64_t B)
{
    sig::WordSet& w = const_cast<sig::WordSet&>(cw);     // the cache is logically mutable
    const int64_t n_units = jit_units(w, dir, B);
    const int wgw = jit_wg_waves(w), tile = jit_tile_for(w, dir);
    std::lock_guard<std::mutex> lock(g_jit_mutex);
    for (auto* e : w.jit[dir])
        if (e->n_units == n_units && e->wg_waves == wgw && e->tile == tile) return e;
    auto* e = new (std::nothrow) sig::WordSet::JitEntry;
    if (!e) return nullptr;
    try {
        e->n_units = n_units;
        e->wg_waves = wgw;
        e->tile = tile;
        if (dir == 0) sig::build_plan_balanced(w, n_units, 320, false, 1, 1, e->plan);
        else sig::build_plan_balanced(w, n_units, 160, true, 6, 9, e->plan);
        e->kernel = new sig::JitKernel;
        w.jit[dir].push_back(e);
    } catch (const std::bad_alloc&) {
        delete e;
        return nullptr;
    }
    return e;
}

// Source of the specialised kernel of an entry; fills nw / tile.
std::string jit_source(const sig::WordSet& w, int dir, const sig::Plan& p, int& nw, int& tile)
{
    // Four wavefronts per workgroup = one per SIMD, so a workgroup's registers fit whatever a unit needs.
    nw = (int)std::min<size_t>((size_t)jit_wg_waves(w), std::max<size_t>(1, p.units.size()));
    tile = jit_tile_for(w, dir);
    return dir ? sig::jit_backward_source(w, p, nw, tile) : sig::jit_forward_source(w, p, nw, tile);
}

// What a call may do to get its kernel: compile and load it (ordinary entry points), or only use one that is already
// loaded (the entry point that allocates nothing: loading a code object allocates device memory).
enum class Build { compile_only, compile_and_load, loaded_only };
// Set by ensure_* when a Build::loaded_only call found a kernel that exists but is not compiled or loaded yet.
thread_local bool g_not_ready = false;

// Brings one kernel to the asked state under the kernel's own lock (a compilation of seconds does not hold up calls
// on other word sets or kernels); `source` is called at most once per kernel.
template <class MakeSource>
sig::JitKernel* bring_up(sig::JitKernel* k, Build how, const char* name, MakeSource source)
{
    std::lock_guard<std::mutex> lock(k->m);
    if (how == Build::loaded_only) {
        if (k->tried && !k->ok) return nullptr;          // specialisation failed earlier: the fallback kernels run
        if (!k->fn) { g_not_ready = true; return nullptr; }
        return k;
    }
    std::string src;
    if (!k->tried) {
        k->tried = true;
        try {
            src = source(*k);
            (void)sig::jit_compile(src, name, *k);
        } catch (const std::bad_alloc&) { k->ok = false; }
    }
    if (!k->ok) return nullptr;
    if (how == Build::compile_and_load && !k->fn && sig::jit_load(*k) != hipSuccess) {
        // a code object from the disk cache that does not load is removed and compiled afresh, once
        bool again = false;
        if (!k->cache_file.empty()) {
            try {
                if (src.empty()) src = source(*k);
                again = sig::jit_compile(src, name, *k, false) == 0 && sig::jit_load(*k) == hipSuccess;
            } catch (const std::bad_alloc&) { again = false; }
        }
        if (!again) {
            k->ok = false;
            return nullptr;
        }
    }
    return k;
}

// Kernel for (direction, batch size) in the asked state, or nullptr if specialisation is off or failed.
// Compilation happens once per entry; the outcome is remembered.  *plan receives the entry's plan.
sig::JitKernel* ensure_jit(const sig::WordSet& cw, int dir, int64_t B, Build how, const sig::Plan** plan = nullptr)
{
    if (!jit_enabled(cw)) return nullptr;
    sig::WordSet::JitEntry* e = jit_entry(cw, dir, B);
    if (!e) return nullptr;
    if (plan) *plan = &e->plan;
    return bring_up(e->kernel, how, dir ? "sig_bwd_jit" : "sig_fwd_jit",
                    [&](sig::JitKernel& k) { return jit_source(cw, dir, e->plan, k.nw, k.tile); });
}

// bytes of the transposed increments the specialised kernels read: [groups][Lpad][d][64] floats
int64_t jit_lpad(const sig::WordSet& w, int64_t n_points, int dir)
{
    const int64_t T = jit_tile_for(w, dir), L = n_points - 1;
    return (L + T - 1) / T * T;
}
size_t jit_dxt_bytes(const sig::WordSet& w, int64_t B, int64_t n_points, int dir)
{
    const size_t n = (size_t)((B + 63) / 64) * (size_t)jit_lpad(w, n_points, dir) * (size_t)w.d * 64 * sizeof(float);
    return (n + 255) & ~(size_t)255;
}

hipError_t launch_jit_forward(sig::JitKernel& k, const sig::Plan& p, const float* dxT, int64_t B, int64_t ntiles, float* coeffs,
                              int64_t nW, hipStream_t st)
{
    long lB = (long)B, lT = (long)ntiles, lW = (long)nW;
    void* args[] = {(void*)&dxT, (void*)&lB, (void*)&lT, (void*)&coeffs, (void*)&lW};
    const unsigned gx = (unsigned)((p.units.size() + (size_t)k.nw - 1) / (size_t)k.nw);
    const unsigned gy = (unsigned)((B + 63) / 64);
    return hipModuleLaunchKernel(k.fn, gx, gy, 1, (unsigned)k.nw * 64, 1, 1, 0, st, args, nullptr);
}

// B rows; with C > 1 they are the C time chunks of B / C paths, whose last chunks read row (path) of coeffs_last and
// grad_last and the others row (path * C + chunk) of coeffs and grad.  C = 1: coeffs and grad hold a row per path.
hipError_t launch_jit_backward(sig::JitKernel& k, const sig::Plan& p, const float* dxT, const float* coeffs, const float* grad,
                               int64_t B, int64_t L, int64_t ntiles, int64_t nW, float* gdx, hipStream_t st,
                               const float* coeffs_last = nullptr, const float* grad_last = nullptr, int64_t C = 1)
{
    long lB = (long)B, lL = (long)L, lT = (long)ntiles, lW = (long)nW, lC = (long)C;
    if (C <= 1) { coeffs_last = coeffs; grad_last = grad; lC = 1; }
    void* args[] = {(void*)&dxT, (void*)&coeffs, (void*)&grad, (void*)&lB, (void*)&lL, (void*)&lT, (void*)&lW, (void*)&gdx,
                    (void*)&coeffs_last, (void*)&grad_last, (void*)&lC};
    const unsigned gx = (unsigned)((p.units.size() + (size_t)k.nw - 1) / (size_t)k.nw);
    const unsigned gy = (unsigned)((B + 63) / 64);
    return hipModuleLaunchKernel(k.fn, gx, gy, 1, (unsigned)k.nw * 64, 1, 1, 0, st, args, nullptr);
}

int bwd_tile_steps(int d) { return std::max(1, std::min(16, 32 / std::max(d, 1))); }

// ---- time chunks of word sets closed under suffixes: rows = (path, chunk) pairs of the specialised kernels ------------
sig::WordTables word_tables(const sig::WordSet& w)
{
    sig::WordTables t;
    const unsigned char* base = (const unsigned char*)w.dev;
    t.prod_pairs = (const uint32_t*)(base + w.dev_prod_off);
    t.adj_pairs = (const uint32_t*)(base + w.dev_adj_pairs_off);
    t.adj_key = (const uint32_t*)(base + w.dev_adj_key_off);
    t.adj_groups = (int)(w.adj_pairs.size() / 256);
    for (int n = 0; n <= w.max_len + 1; ++n) {
        t.level_start[n] = w.level_start[(size_t)n];
        t.tail_off[n] = w.tail_off[(size_t)n];
    }
    t.N = w.max_len;
    t.W = (int)w.size();
    return t;
}
// Both kernels for B * C rows, compiled and loaded, or false: then the checkpointed calls run as the plain ones (the
// outcome of a compilation is remembered, so the forward and the backward call of a pair decide alike).
bool words_kernels(const sig::WordSet& w, int64_t rows, sig::JitKernel** fwd, const sig::Plan** fplan, sig::JitKernel** bwd,
                   const sig::Plan** bplan)
{
    *fwd = ensure_jit(w, 0, rows, Build::compile_and_load, fplan);
    *bwd = *fwd ? ensure_jit(w, 1, rows, Build::compile_and_load, bplan) : nullptr;
    return *fwd && *bwd;
}
size_t words_forward_ckpt_workspace(const sig::WordSet& w, int64_t B, const Chunks& ch)
{
    return jit_dxt_bytes(w, B * ch.C, ch.Lc + 1, 0);
}
// increment gradients and increments of all rows in the transposed layout | boundary adjoints (for more than two chunks
// first what follows every chunk, overwritten in place) | for more than two chunks: signatures at the chunk ends
// The chunked forward pass: transposed increments of all (path, chunk) rows, their signatures into Sc [B][C][|W|], the
// product of every path's chunk signatures into coeffs (nullptr: the chunk signatures alone).
hipError_t words_forward_chunked(const sig::WordSet& w, const float* path, int64_t B, int64_t n_points, const Chunks& ch,
                                 sig::JitKernel& fk, const sig::Plan& fp, float* dxT, float* Sc, float* coeffs, hipStream_t st)
{
    sig::WindowList rows;
    rows.K = ch.C; rows.max_len = ch.Lc;
    const int64_t Lpad = jit_lpad(w, ch.Lc + 1, 0);
    hipError_t e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, nullptr, st, rows);
    if (e != hipSuccess) return e;
    hipEvent_t* pe = g_prof.next(0);
    if (pe) (void)hipEventRecord(pe[0], st);
    e = launch_jit_forward(fk, fp, dxT, B * ch.C, Lpad / fk.tile, Sc, w.size(), st);
    if (pe) (void)hipEventRecord(pe[1], st);
    if (e == hipSuccess && coeffs) e = sig::words_scan(word_tables(w), Sc, B, (int)ch.C, false, nullptr, coeffs, st);
    return e;
}
size_t words_backward_ckpt_workspace(const sig::WordSet& w, int64_t B, const Chunks& ch)
{
    return 2 * jit_dxt_bytes(w, B * ch.C, ch.Lc + 1, 1) + (ch.C == 2 ? 1 : 2) * chunk_array_bytes(w, B, ch.C);
}
// The backward pass over the (path, chunk) rows of a suffix-closed set, from the chunk signatures Sc [B][C][|W|]:
// boundary adjoints (and, beyond two chunks, the signatures at the chunk ends) from products over the set, one launch
// of the specialised kernel over all rows, chain rule.  workspace: words_backward_ckpt_workspace bytes.
hipError_t words_backward_chunked(const sig::WordSet& w, const float* path, const float* coeffs, const float* grad_coeffs,
                                  const float* Sc, const Chunks& ch, int64_t B, int64_t n_points, float* grad_path, void* workspace,
                                  sig::JitKernel& bk, const sig::Plan& bp, hipStream_t st)
{
    sig::WindowList rows;
    rows.K = ch.C; rows.max_len = ch.Lc;
    const size_t t_bytes = jit_dxt_bytes(w, B * ch.C, ch.Lc + 1, 1), nb = chunk_array_bytes(w, B, ch.C);
    float* gdx = (float*)workspace;
    float* dxT = (float*)((unsigned char*)workspace + t_bytes);
    float* Abar = (float*)((unsigned char*)workspace + 2 * t_bytes);
    const float* Pfx = Sc;
    const sig::WordTables tab = word_tables(w);
    const int64_t Lpad = jit_lpad(w, ch.Lc + 1, 1);
    // rows of one path share the points between their chunks: the chain rule adds into grad_path, which the adjoint
    // kernel clears on the way
    const int64_t n_gp = B * n_points * w.d;
    hipError_t e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, gdx, st, rows);
    if (ch.C == 2) {
        // two chunks: the signature at the end of the first is the first chunk's own, what follows it the second's
        // (row c + 1 of the chunk signatures, read as row c of an array that starts one row later)
        if (e == hipSuccess) e = sig::words_adjoint(tab, grad_coeffs, Sc + w.size(), B, 2, Abar, grad_path, n_gp, st);
    } else {
        float* P = (float*)((unsigned char*)workspace + 2 * t_bytes + nb);
        if (e == hipSuccess) e = sig::words_scan_both(tab, Sc, B, (int)ch.C, P, Abar, st);
        if (e == hipSuccess) e = sig::words_adjoint(tab, grad_coeffs, Abar, B, (int)ch.C, Abar, grad_path, n_gp, st);   // in place, row by row
        Pfx = P;
    }
    if (e != hipSuccess) return e;
    hipEvent_t* pe = g_prof.next(1);
    if (pe) (void)hipEventRecord(pe[0], st);
    // the rows of the last chunk are the caller's terminal signature and gradient themselves
    e = launch_jit_backward(bk, bp, dxT, Pfx, Abar, B * ch.C, ch.Lc, Lpad / bk.tile, w.size(), gdx, st, coeffs, grad_coeffs, ch.C);
    if (pe) (void)hipEventRecord(pe[1], st);
    if (e != hipSuccess) return e;
    return sig::grad_points_transposed(gdx, B, n_points, w.d, Lpad, grad_path, st, rows);
}
// sig_backward on a suffix-closed set recomputes the chunk signatures and takes the same route where that still wins:
// from four chunks on by the rule of the checkpointed calls (measured: 64 paths x 4,096 segments 2.36 -> 0.62 ms,
// 512 x 2,048 1.57 -> 1.24 ms; with two chunks the second forward pass eats the gain).
// workspace: | backward part (its first bytes serve the forward's transposed increments before) | chunk signatures |
bool words_backward_recomputes(const sig::WordSet& w, const Chunks& ch) { return w.kind != 0 && ch.C >= 4; }
size_t words_backward_recompute_first(const sig::WordSet& w, int64_t B, const Chunks& ch)
{
    return std::max(words_backward_ckpt_workspace(w, B, ch), words_forward_ckpt_workspace(w, B, ch));
}
size_t words_backward_recompute_workspace(const sig::WordSet& w, int64_t B, const Chunks& ch)
{
    return words_backward_recompute_first(w, B, ch) + chunk_array_bytes(w, B, ch.C);
}

// ---- full truncations without a register-resident kernel of their own: lanes = words -----------------------
// Lanes = paths needs 64 paths per wavefront and a compilation that grows with the word set (minutes beyond a few
// ten thousand words); lanes = words fills the wavefronts from a single path on and compiles in about a second per
// shape.  Taken whenever the words of a path fill at least half a wavefront; the option "lanes" = 0 switches it off, = 1 takes
// it for every shape it is defined for.
int lanes_levels_asked(const sig::WordSet& w)             // testing knob: 1 or 2 levels below the lane's word
{
    return w.opt.lanes_levels == 1 || w.opt.lanes_levels == 2 ? w.opt.lanes_levels : 0;
}
sig::LanesShape lanes_shape_for(const sig::WordSet& w, int dir, int64_t B)
{
    sig::LanesShape s = sig::lanes_shape(w.d, w.depth, dir != 0, B, lanes_levels_asked(w));
    if (!s.ok) s = sig::lanes_shape(w.d, w.depth, dir != 0, B, 0);
    return s;
}

bool use_lanes(const sig::WordSet& w, int64_t B)
{
    if (w.kind != 0 || !jit_enabled(w)) return false;
    const int f = w.opt.lanes;
    if (f == 0) return false;
    const sig::LanesShape s = lanes_shape_for(w, 0, B), sb = lanes_shape_for(w, 1, B);
    if (!s.ok || !sb.ok || B * std::max(s.waves, sb.waves) > (int64_t)0x7fffffff) return false;
    return f == 1 || std::min(s.lanes, sb.lanes) >= 32;
}

sig::JitKernel* ensure_lanes(const sig::WordSet& cw, int dir, const sig::LanesShape& s, Build how)
{
    sig::WordSet& w = const_cast<sig::WordSet&>(cw);     // the cache is logically mutable
    sig::JitKernel* k = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_jit_mutex);
        sig::JitKernel*& slot = w.lanes[dir][s.R - 1];
        if (!slot) slot = new (std::nothrow) sig::JitKernel;
        k = slot;
    }
    if (!k) return nullptr;
    // everything but the levels per lane follows from (d, depth, direction): one kernel per slot
    return bring_up(k, how, dir ? "sig_bwd_lanes" : "sig_fwd_lanes", [&](sig::JitKernel& kk) {
        kk.nw = s.nwb;
        kk.tile = s.T;
        return sig::lanes_source(w.d, w.depth, s, dir != 0);
    });
}

// rows: the B paths, or with a window list the B * K (path, window) pairs, read straight from the path
hipError_t launch_lanes(sig::JitKernel& k, const sig::LanesShape& s, const float* path, const float* coeffs_in, const float* grad,
                        int64_t B, int64_t n_points, float* out, hipStream_t st, const sig::WindowList& wl = sig::WindowList())
{
    long lB = (long)B, lP = (long)n_points, lK = (long)wl.K, lM = (long)wl.max_len;
    const int64_t* win = wl.win;
    const int64_t rows = B * (wl.win ? wl.K : 1);
    const int64_t blocks = (rows * s.waves + k.nw - 1) / k.nw;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (grad) {
        void* args[] = {(void*)&path, (void*)&coeffs_in, (void*)&grad, (void*)&lB, (void*)&lP, (void*)&out, (void*)&win, (void*)&lK,
                        (void*)&lM};
        return hipModuleLaunchKernel(k.fn, (unsigned)blocks, 1, 1, (unsigned)k.nw * 64, 1, 1, 0, st, args, nullptr);
    }
    void* args[] = {(void*)&path, (void*)&lB, (void*)&lP, (void*)&out, (void*)&win, (void*)&lK, (void*)&lM};
    return hipModuleLaunchKernel(k.fn, (unsigned)blocks, 1, 1, (unsigned)k.nw * 64, 1, 1, 0, st, args, nullptr);
}
}  // namespace

extern "C" {

int sig_wordset_build_truncated(int d, int depth, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_truncated(d, depth, &w), w, out);
}

int sig_wordset_build_anisotropic(int d, const double* weights, double cutoff, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_anisotropic(d, weights, cutoff, &w), w, out);
}

int sig_wordset_build(int d, const int32_t* letters, const int64_t* offsets, int64_t n_words, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_list(d, letters, offsets, n_words, &w), w, out);
}

int sig_wordset_build_graph(int d, const int32_t* edges, int64_t n_edges, int depth, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_graph(d, edges, n_edges, depth, &w), w, out);
}

int sig_wordset_build_leadlag_sparse(int d, int depth, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_leadlag_sparse(d, depth, &w), w, out);
}

int sig_wordset_build_logsig(int d, int depth, sig_wordset** out)
{
    if (!out) return SIG_EINVAL;
    sig::WordSet* w = nullptr;
    return finish_build(sig::build_logsig(d, depth, &w), w, out);
}

int sig_wordset_set_option(sig_wordset* ws, const char* name, int value)
{
    if (!ws || !name) return SIG_EINVAL;
    for (const OptionName& o : kOptions)
        if (std::strcmp(o.name, name) == 0) {
            ws->opt.*(o.field) = value;
            return SIG_OK;
        }
    return SIG_EINVAL;
}

int sig_wordset_get_option(const sig_wordset* ws, const char* name, int* value)
{
    if (!ws || !name || !value) return SIG_EINVAL;
    for (const OptionName& o : kOptions)
        if (std::strcmp(o.name, name) == 0) {
            *value = W(ws)->opt.*(o.field);
            return SIG_OK;
        }
    return SIG_EINVAL;
}

int64_t sig_wordset_n_lyndon(const sig_wordset* ws) { return ws ? W(ws)->n_lyndon : -1; }

int sig_logsig_forward(const sig_wordset* ws, const float* coeffs, int64_t B, float* logsig, void* stream)
{
    if (!ws || B < 0) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    if (w.n_lyndon <= 0) return SIG_EUNSUPPORTED;
    if (!w.dev) return SIG_ENOTUPLOADED;
    if (B == 0) return SIG_OK;
    if (!coeffs || !logsig) return SIG_EINVAL;
    const unsigned char* base = (const unsigned char*)w.dev;
    hipError_t e = sig::logsig_forward(coeffs, B, w.size(), (const int32_t*)(base + w.lyn_len_off),
                                       (const int32_t*)(base + w.lyn_sub_off), w.n_lyndon, w.lyn_stride, w.depth, logsig,
                                       (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

size_t sig_logsig_backward_workspace_bytes(const sig_wordset* ws, int64_t B)
{
    if (!ws || B <= 0 || W(ws)->n_lyndon <= 0) return 0;
    return ((size_t)B * (size_t)W(ws)->n_lyndon * (size_t)W(ws)->lyn_pairs * sizeof(float) + 255) & ~(size_t)255;
}

int sig_logsig_backward(const sig_wordset* ws, const float* coeffs, const float* grad_logsig, int64_t B, float* grad_coeffs,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ws || B < 0) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    if (w.n_lyndon <= 0) return SIG_EUNSUPPORTED;
    if (!w.dev) return SIG_ENOTUPLOADED;
    if (B == 0) return SIG_OK;
    if (!coeffs || !grad_logsig || !grad_coeffs) return SIG_EINVAL;
    if (!workspace || workspace_bytes < sig_logsig_backward_workspace_bytes(ws, B)) return SIG_EWORKSPACE;
    const unsigned char* base = (const unsigned char*)w.dev;
    hipError_t e = sig::logsig_backward(coeffs, grad_logsig, B, w.size(), (const int32_t*)(base + w.lyn_len_off),
                                        (const int32_t*)(base + w.lyn_sub_off), w.n_lyndon, w.lyn_stride, w.depth, w.lyn_pairs,
                                        (const int32_t*)(base + w.lyn_inv_off_off), (const int32_t*)(base + w.lyn_inv_ent_off),
                                        (float*)workspace, grad_coeffs, w.opt.logsig_gather != 0, (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_leadlag_transform(const float* path, int64_t B, int64_t n_points, int d, float* out, void* stream)
{
    if (B < 0 || n_points < 1 || d < 1) return SIG_EINVAL;
    if (B == 0) return SIG_OK;
    if (!path || !out) return SIG_EINVAL;
    hipError_t e = sig::leadlag(path, B, n_points, d, out, (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_leadlag_backward(const float* grad_out, int64_t B, int64_t n_points, int d, float* grad_path, void* stream)
{
    if (B < 0 || n_points < 1 || d < 1) return SIG_EINVAL;
    if (B == 0) return SIG_OK;
    if (!grad_out || !grad_path) return SIG_EINVAL;
    hipError_t e = sig::leadlag_backward(grad_out, B, n_points, d, grad_path, (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

void sig_wordset_free(sig_wordset* ws) { delete static_cast<sig::WordSet*>(ws); }

int64_t sig_wordset_size(const sig_wordset* ws) { return ws ? W(ws)->size() : -1; }
int sig_wordset_dim(const sig_wordset* ws) { return ws ? W(ws)->d : -1; }
int sig_wordset_max_len(const sig_wordset* ws) { return ws ? W(ws)->max_len : -1; }
int64_t sig_wordset_n_user(const sig_wordset* ws) { return ws ? (int64_t)W(ws)->user_index.size() : -1; }
const int32_t* sig_wordset_parent(const sig_wordset* ws) { return ws ? W(ws)->parent.data() : nullptr; }
const int32_t* sig_wordset_letter(const sig_wordset* ws) { return ws ? W(ws)->letter.data() : nullptr; }
const int32_t* sig_wordset_level_start(const sig_wordset* ws) { return ws ? W(ws)->level_start.data() : nullptr; }
const int64_t* sig_wordset_user_index(const sig_wordset* ws)
{
    return (ws && !W(ws)->user_index.empty()) ? W(ws)->user_index.data() : nullptr;
}
int sig_wordset_suffix_closed(const sig_wordset* ws) { return ws ? (W(ws)->suffix_closed ? 1 : 0) : -1; }
const int32_t* sig_wordset_tail_table(const sig_wordset* ws, const int32_t** tail_off)
{
    if (!ws || !W(ws)->suffix_closed) return nullptr;
    if (tail_off) *tail_off = W(ws)->tail_off.data();
    return W(ws)->tail_tab.data();
}
int64_t sig_wordset_term_tables(const sig_wordset* ws, const uint32_t** prod_pairs, const uint32_t** adj_pairs,
                                const uint32_t** adj_key, int64_t* n_adj)
{
    if (!ws || !W(ws)->pair_tables) return -1;
    if (prod_pairs) *prod_pairs = W(ws)->prod_pairs.data();
    if (adj_pairs) *adj_pairs = W(ws)->adj_pairs.data();
    if (adj_key) *adj_key = W(ws)->adj_key.data();
    if (n_adj) *n_adj = (int64_t)W(ws)->adj_pairs.size();
    return (int64_t)W(ws)->prod_pairs.size();
}
int64_t sig_wordset_min_fma_per_step(const sig_wordset* ws) { return ws ? W(ws)->min_fma : -1; }

int64_t sig_wordset_kernel_fma_per_step(const sig_wordset* ws, int backward)
{
    if (!ws || !W(ws)->kernels_supported) return -1;
    // reported for the finest variant unless a launch picked another one; forward count of
    // multiply-adds, the backward kernels issue about 3 per leaf pair and 4.5 per inner pair
    const auto& pl = W(ws)->plans[backward ? 1 : 0];
    return pl.empty() ? -1 : pl.front().fma_per_step;
}

int sig_wordset_plan_count(const sig_wordset* ws, int backward)
{
    return ws ? (int)W(ws)->plans[backward ? 1 : 0].size() : -1;
}

int sig_wordset_plan_get(const sig_wordset* ws, int backward, int variant, const int32_t** units, int64_t* n_units,
                         const uint32_t** ops, int64_t* n_ops, const int32_t** slot_word, int64_t* n_slots,
                         int64_t* fma_per_step)
{
    if (!ws) return SIG_EINVAL;
    const auto& pl = W(ws)->plans[backward ? 1 : 0];
    if (variant < 0 || variant >= (int)pl.size()) return SIG_EINVAL;
    const sig::Plan& p = pl[(size_t)variant];
    static_assert(sizeof(sig::UnitDesc) == 4 * sizeof(int32_t), "UnitDesc is four int32");
    if (units) *units = reinterpret_cast<const int32_t*>(p.units.data());
    if (n_units) *n_units = (int64_t)p.units.size();
    if (ops) *ops = p.ops.data();
    if (n_ops) *n_ops = (int64_t)p.ops.size();
    if (slot_word) *slot_word = p.slot_word.data();
    if (n_slots) *n_slots = (int64_t)p.slot_word.size();
    if (fma_per_step) *fma_per_step = p.fma_per_step;
    return SIG_OK;
}

int sig_wordset_jit_plan_get(sig_wordset* ws, int backward, int64_t B, const int32_t** units, int64_t* n_units,
                             const uint32_t** ops, int64_t* n_ops, const int32_t** slot_word, int64_t* n_slots,
                             int64_t* fma_per_step)
{
    if (!ws || B < 1) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    if (!w.kernels_supported || w.size() == 0) return SIG_EUNSUPPORTED;
    sig::WordSet::JitEntry* e = jit_entry(w, backward ? 1 : 0, B);
    if (!e) return SIG_ENOMEM;
    const sig::Plan& p = e->plan;
    if (units) *units = reinterpret_cast<const int32_t*>(p.units.data());
    if (n_units) *n_units = (int64_t)p.units.size();
    if (ops) *ops = p.ops.data();
    if (n_ops) *n_ops = (int64_t)p.ops.size();
    if (slot_word) *slot_word = p.slot_word.data();
    if (n_slots) *n_slots = (int64_t)p.slot_word.size();
    if (fma_per_step) *fma_per_step = p.fma_per_step;
    return SIG_OK;
}

int sig_wordset_jit_prepare(sig_wordset* ws, int backward, int64_t B)
{
    if (!ws || B < 1) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    const int dir = backward ? 1 : 0;
    if (!jit_enabled(w)) return SIG_EUNSUPPORTED;
    if (dir == 0 ? use_trunc_forward(w, B) : use_trunc_backward(w, B)) return SIG_EUNSUPPORTED;
    if (use_lanes(w, B)) return ensure_lanes(w, dir, lanes_shape_for(w, dir, B), Build::compile_only) ? SIG_OK : SIG_EJIT;
    return ensure_jit(w, dir, B, Build::compile_only) ? SIG_OK : SIG_EJIT;
}

size_t sig_wordset_jit_source(sig_wordset* ws, int backward, int64_t B, char* buf, size_t n)
{
    if (!ws || B < 1) return 0;
    const sig::WordSet& w = *W(ws);
    const int dir = backward ? 1 : 0;
    if (!jit_enabled(w)) return 0;
    std::string src;
    if (use_lanes(w, B)) {
        src = sig::lanes_source(w.d, w.depth, lanes_shape_for(w, dir, B), dir != 0);
    } else {
        sig::WordSet::JitEntry* e = jit_entry(w, dir, B);
        if (!e) return 0;
        int nw = 0, tile = 0;
        src = jit_source(w, dir, e->plan, nw, tile);
    }
    if (buf && n > 0) {
        const size_t c = std::min(n - 1, src.size());
        std::memcpy(buf, src.data(), c);
        buf[c] = 0;
    }
    return src.size();
}

size_t sig_wordset_device_bytes(const sig_wordset* ws) { return ws ? W(ws)->image.size() : 0; }

int sig_wordset_upload(sig_wordset* ws, void* dev_buf, size_t dev_bytes, void* stream)
{
    if (!ws || !dev_buf) return SIG_EINVAL;
    if (dev_bytes < ws->image.size()) return SIG_EWORKSPACE;
    if (((uintptr_t)dev_buf & 255) != 0) return SIG_EINVAL;
    hipError_t e = hipMemcpyAsync(dev_buf, ws->image.data(), ws->image.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    ws->dev = dev_buf;
    (void)hipGetDevice(&ws->dev_id);
    return SIG_OK;
}

size_t sig_forward_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    if (!ws || B <= 0 || n_points <= 1) return 0;
    const sig::WordSet& w = *W(ws);
    if (use_trunc_forward(w, B)) {
        const Chunks ch = trunc_chunks(w, 0, B, n_points);
        return ch.C > 1 ? forward_chunk_arrays(w, ch.C) * chunk_array_bytes(w, B, ch.C) : 0;
    }
    if (!jit_enabled(w)) return 0;
    size_t n = jit_dxt_bytes(w, B, n_points, 0);
    if (w.kind != 0) {
        // sets closed under suffixes: time chunks as in the checkpointed calls, the chunk signatures in the workspace
        const Chunks ch = checkpoint_chunks(w, B, n_points);
        if (ch.C >= 2) n = std::max(n, words_forward_ckpt_workspace(w, B, ch) + chunk_array_bytes(w, B, ch.C));
    }
    return n;
}

// what sig_backward needs; own_chunks = false: when it takes no time chunks of its own (sig_backward_static)
static size_t backward_workspace(const sig_wordset* ws, int64_t B, int64_t n_points, bool own_chunks)
{
    if (!ws || B <= 0 || n_points <= 1) return 0;
    const sig::WordSet& w = *W(ws);
    size_t n = (size_t)B * (size_t)(n_points - 1) * (size_t)w.d * sizeof(float);
    n = (n + 255) & ~(size_t)255;                                   // gradient with respect to the increments
    if (use_trunc_backward(w, B)) {
        const BwdShape ch = trunc_backward_shape(w, B, n_points, own_chunks);
        if (ch.C > 1 && !ch.fused) n += 4 * chunk_array_bytes(w, B, ch.C);   // chunk signatures, prefixes, suffixes, adjoints
    } else if (jit_enabled(w)) {
        // the specialised kernels keep the increment gradients in the (padded) layout of their transposed increments
        const size_t t = jit_dxt_bytes(w, B, n_points, 1);
        n = std::max(n, t) + t;
    }
    return n;
}

size_t sig_backward_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    size_t n = backward_workspace(ws, B, n_points, true);
    if (n == 0) return 0;
    const sig::WordSet& w = *W(ws);
    if (w.kind != 0 && jit_enabled(w)) {
        const Chunks ch = checkpoint_chunks(w, B, n_points);
        if (words_backward_recomputes(w, ch)) n = std::max(n, words_backward_recompute_workspace(w, B, ch));
    }
    return n;
}

static int check_common(const sig_wordset* ws, const void* path, int64_t B, int64_t n_points)
{
    if (!ws) return SIG_EINVAL;
    if (B < 0 || n_points < 1) return SIG_EINVAL;
    if (B > 0 && !path) return SIG_EINVAL;
    if (!W(ws)->kernels_supported) return SIG_EUNSUPPORTED;
    if (!W(ws)->dev) return SIG_ENOTUPLOADED;
    if (B > (int64_t)65535 * 64) return SIG_ETOOLARGE;
    return SIG_OK;
}

// sig_forward; word_chunks = false keeps a suffix-closed set from taking time chunks of its own (the checkpointed call
// that falls back to this one has sized its workspace for whole paths)
static int forward_impl(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, float* coeffs, void* workspace,
                        size_t workspace_bytes, void* stream, bool word_chunks)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!coeffs) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    hipStream_t st = (hipStream_t)stream;
    if (n_points == 1) {
        hipError_t e = sig::fill_zero(coeffs, B * w.size(), st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    CallTimer whole(0, st);
    if (use_trunc_forward(w, B)) {
        if (const int64_t C = trunc_forward_fused_chunks(w, B, n_points, coeffs)) {
            const int64_t Lc = (n_points - 1 + C - 1) / C;
            hipEvent_t* pe = g_prof.next(0);
            if (pe) (void)hipEventRecord(pe[0], st);
            hipError_t e = sig::trunc_forward_tails_fused(w.d, w.depth, path, B, n_points, C, Lc, coeffs, st);
            if (pe) (void)hipEventRecord(pe[1], st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
        const Chunks ch = trunc_chunks(w, 0, B, n_points);
        float* Sc = coeffs;
        float* Pfx = nullptr;
        if (ch.C > 1) {
            const size_t nb = chunk_array_bytes(w, B, ch.C);
            if (!workspace || workspace_bytes < forward_chunk_arrays(w, ch.C) * nb) return SIG_EWORKSPACE;
            if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)coeffs & 15) != 0) return SIG_EINVAL;
            Sc = (float*)workspace;
            if (forward_chunk_arrays(w, ch.C) > 1) Pfx = (float*)((unsigned char*)workspace + nb);
        }
        hipEvent_t* pe = g_prof.next(0);
        if (pe) (void)hipEventRecord(pe[0], st);
        hipError_t e = sig::trunc_forward(w.d, w.depth, path, B, n_points, ch.C, ch.Lc, Sc, st);
        if (pe) (void)hipEventRecord(pe[1], st);
        if (e == hipSuccess && ch.C > 1)
            e = sig::chunk_scan(w.d, w.depth, Sc, Pfx, nullptr, nullptr, coeffs, nullptr, nullptr, B, (int)ch.C, nullptr, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    if (use_lanes(w, B)) {
        const sig::LanesShape ls = lanes_shape_for(w, 0, B);
        if (sig::JitKernel* lk = ensure_lanes(w, 0, ls, Build::compile_and_load)) {
            hipEvent_t* pe = g_prof.next(0);
            if (pe) (void)hipEventRecord(pe[0], st);
            hipError_t e = launch_lanes(*lk, ls, path, nullptr, nullptr, B, n_points, coeffs, st);
            if (pe) (void)hipEventRecord(pe[1], st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    if (w.kind != 0 && word_chunks) {
        // sets closed under suffixes: the time chunks of the checkpointed calls, with the chunk signatures in the workspace
        const Chunks ch = checkpoint_chunks(w, B, n_points);
        const sig::Plan* cp = nullptr;
        sig::JitKernel* ck = ch.C >= 2 ? ensure_jit(w, 0, B * ch.C, Build::compile_and_load, &cp) : nullptr;
        if (ck) {
            if (!workspace || workspace_bytes < sig_forward_workspace_bytes(ws, B, n_points)) return SIG_EWORKSPACE;
            if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
            float* dxT = (float*)workspace;
            float* Sc = (float*)((unsigned char*)workspace + words_forward_ckpt_workspace(w, B, ch));
            hipError_t e = words_forward_chunked(w, path, B, n_points, ch, *ck, *cp, dxT, Sc, coeffs, st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    const sig::Plan* jp = nullptr;
    if (sig::JitKernel* jk = ensure_jit(w, 0, B, Build::compile_and_load, &jp)) {
        if (!workspace || workspace_bytes < jit_dxt_bytes(w, B, n_points, 0)) return SIG_EWORKSPACE;
        if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
        float* dxT = (float*)workspace;
        const int64_t Lpad = jit_lpad(w, n_points, 0);
        hipError_t e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, nullptr, st);
        if (e != hipSuccess) return hip_fail(e);
        hipEvent_t* pe = g_prof.next(0);
        if (pe) (void)hipEventRecord(pe[0], st);
        e = launch_jit_forward(*jk, *jp, dxT, B, Lpad / jk->tile, coeffs, w.size(), st);
        if (pe) (void)hipEventRecord(pe[1], st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    const int v = pick_variant(w, 0, B);
    const sig::Plan& p = w.plans[0][(size_t)v];
    const auto& po = w.offsets[0][(size_t)v];
    const unsigned char* base = (const unsigned char*)w.dev;
    sig::GenericArgs a;
    a.units = (const sig::UnitDesc*)(base + po.units);
    a.ops = (const uint32_t*)(base + po.ops);
    a.slot_word = (const int32_t*)(base + po.slots);
    a.n_units = (int64_t)p.units.size();
    a.max_slots = p.max_slots;
    a.path = path; a.B = B; a.P = n_points; a.d = w.d; a.nW = w.size();
    a.coeffs = coeffs;
    hipEvent_t* pe = g_prof.next(0);
    if (pe) (void)hipEventRecord(pe[0], st);
    hipError_t e = sig::generic_forward(a, w.max_len, st);
    if (pe) (void)hipEventRecord(pe[1], st);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_forward(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, float* coeffs, void* workspace,
                size_t workspace_bytes, void* stream)
{
    return forward_impl(ws, path, B, n_points, coeffs, workspace, workspace_bytes, stream, true);
}

// sig_backward and sig_backward_static: the same kernels on the caller's workspace or on the static scratch array;
// `how` says whether a run-time specialised kernel may be compiled and loaded by this call.
static size_t gdx_bytes_of(const sig::WordSet& w, int64_t B, int64_t n_points)
{
    return ((size_t)B * (size_t)(n_points - 1) * (size_t)w.d * sizeof(float) + 255) & ~(size_t)255;
}

// Backward over the C time chunks whose signatures the forward pass left in ckpt [B][C][|W|]: signature and adjoint at
// the end of every chunk from products of the chunk signatures, then all (path, chunk) rows in one launch.
static int backward_checkpointed(const sig::WordSet& w, const float* path, const float* coeffs, const float* grad_coeffs,
                                 const float* ckpt, const Chunks& ch, int64_t B, int64_t n_points, float* grad_path,
                                 void* workspace, hipStream_t st)
{
    if ((((uintptr_t)coeffs | (uintptr_t)grad_coeffs | (uintptr_t)ckpt) & 15) != 0) return SIG_EINVAL;
    const int64_t nW = w.size();
    // workspace: increment gradients | boundary adjoints [B][C - 1][|W|] | for more than two chunks: products from the
    // left and from the right, [B][C][|W|] each
    const size_t gb = gdx_bytes_of(w, B, n_points), nb = chunk_array_bytes(w, B, ch.C), ab = chunk_array_bytes(w, B, ch.C - 1);
    float* gdx = (float*)workspace;
    float* Abar = (float*)((unsigned char*)workspace + gb);
    CallTimer whole(1, st);
    hipError_t e = sig::fill_zero(gdx, B * (n_points - 1) * w.d, st);
    const float* row_coeffs = ckpt;
    if (ch.C == 2) {
        // two chunks: the signature at the end of the first is the first chunk's own, what follows it the second's
        if (e == hipSuccess) e = sig::chunk_adjoint(w.d, w.depth, grad_coeffs, ckpt + nW, Abar, B, 2, true, st);
    } else {
        float* Pfx = (float*)((unsigned char*)workspace + gb + ab);
        float* Q = (float*)((unsigned char*)workspace + gb + ab + nb);
        if (e == hipSuccess)
            e = sig::chunk_scan(w.d, w.depth, ckpt, Pfx, Q, coeffs, nullptr, nullptr, nullptr, B, (int)ch.C, nullptr, st);
        if (e == hipSuccess) e = sig::chunk_adjoint(w.d, w.depth, grad_coeffs, Q, Abar, B, (int)ch.C, true, st);
        row_coeffs = Pfx;
    }
    if (e != hipSuccess) return hip_fail(e);
    hipEvent_t* pe = g_prof.next(1);
    if (pe) (void)hipEventRecord(pe[0], st);
    // the rows of the last chunk are the caller's terminal signature and gradient themselves
    e = sig::trunc_backward(w.d, w.depth, path, row_coeffs, Abar, coeffs, grad_coeffs, B, n_points, ch.C, ch.Lc, gdx, nullptr,
                            w.opt.bwd_tile, st);
    if (pe) (void)hipEventRecord(pe[1], st);
    if (e != hipSuccess) return hip_fail(e);
    e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

static int backward_impl(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                         int64_t n_points, float* grad_path, void* workspace, size_t workspace_bytes, void* stream, Build how,
                         float* residual = nullptr, bool word_chunks = true /* false: no time chunks of its own */)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    if (B == 0) return SIG_OK;
    if (!coeffs || !grad_coeffs || !grad_path) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    hipStream_t st = (hipStream_t)stream;
    if (n_points == 1) {
        hipError_t e = sig::fill_zero(grad_path, B * w.d, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    const size_t need = word_chunks ? sig_backward_workspace_bytes(ws, B, n_points) : backward_workspace(ws, B, n_points, false);
    if (!workspace || workspace_bytes < need) return SIG_EWORKSPACE;
    if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
    float* gdx = (float*)workspace;
    CallTimer whole(1, st);
    if (word_chunks && w.kind != 0 && jit_enabled(w) && !residual) {
        // suffix-closed set, few long paths: chunk signatures recomputed, then the route of the checkpointed call
        const Chunks wc = checkpoint_chunks(w, B, n_points);
        sig::JitKernel *fk, *bk;
        const sig::Plan *fp = nullptr, *bp = nullptr;
        if (words_backward_recomputes(w, wc) && words_kernels(w, B * wc.C, &fk, &fp, &bk, &bp)) {
            float* Sc = (float*)((unsigned char*)workspace + words_backward_recompute_first(w, B, wc));
            hipError_t ce = words_forward_chunked(w, path, B, n_points, wc, *fk, *fp, (float*)workspace, Sc, nullptr, st);
            if (ce == hipSuccess)
                ce = words_backward_chunked(w, path, coeffs, grad_coeffs, Sc, wc, B, n_points, grad_path, workspace, *bk, *bp, st);
            return ce == hipSuccess ? SIG_OK : hip_fail(ce);
        }
    }
    hipError_t e = hipSuccess;
    const bool trunc = use_trunc_backward(w, B);
    BwdShape ch = trunc ? trunc_backward_shape(w, B, n_points, word_chunks) : BwdShape{false, false, 1, n_points - 1};
    if (residual) {                      // reported by the kernels that walk whole paths with several wavefronts per row
        if (!trunc) return SIG_EUNSUPPORTED;
        ch = BwdShape{false, false, 1, n_points - 1};
        e = sig::fill_zero(residual, B, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    // the fused form copies the gradient row with 16-byte loads; rows that are not aligned so take the kernel with
    // four wavefronts per path, which reads word by word
    if (ch.fused && (((uintptr_t)coeffs | (uintptr_t)grad_coeffs) & 15) != 0) ch = BwdShape{false, false, 1, n_points - 1};
    // word sets that may run through the straight-line specialised kernels clear their (larger) array further down
    const bool maybe_jit = !trunc && !use_lanes(w, B) && jit_enabled(w);
    if (!ch.tails && !maybe_jit) {       // the one-wavefront-per-row kernel stores every entry itself
        e = sig::fill_zero(gdx, B * (n_points - 1) * w.d, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (trunc) {
        const float* row_coeffs = coeffs;
        const float* row_grad = grad_coeffs;
        if (ch.C > 1 && !ch.fused) {
            if ((((uintptr_t)coeffs | (uintptr_t)grad_coeffs) & 15) != 0) return SIG_EINVAL;
            // chunk signatures (recomputed: only the terminal signature was kept), then the signature and the
            // adjoint at the end of every chunk
            const size_t gb = ((size_t)B * (size_t)(n_points - 1) * (size_t)w.d * sizeof(float) + 255) & ~(size_t)255;
            const size_t nb = chunk_array_bytes(w, B, ch.C);
            unsigned char* base = (unsigned char*)workspace + gb;
            float* Sc = (float*)base;
            float* Pfx = (float*)(base + nb);
            float* Q = (float*)(base + 2 * nb);
            float* Abar = (float*)(base + 3 * nb);
            e = sig::trunc_forward(w.d, w.depth, path, B, n_points, ch.C, ch.Lc, Sc, st);
            bool adjoints_done = false;
            if (e == hipSuccess)
                e = sig::chunk_scan(w.d, w.depth, Sc, Pfx, Q, coeffs, nullptr, grad_coeffs, Abar, B, (int)ch.C, &adjoints_done, st);
            if (e == hipSuccess && !adjoints_done) e = sig::chunk_adjoint(w.d, w.depth, grad_coeffs, Q, Abar, B, (int)ch.C, false, st);
            if (e != hipSuccess) return hip_fail(e);
            row_coeffs = Pfx;
            row_grad = Abar;
        }
        hipEvent_t* pe = g_prof.next(1);
        if (pe) (void)hipEventRecord(pe[0], st);
        // the one-wavefront-per-row kernel applies the chain rule itself when its rows are whole paths or all
        // chunks of a path share a workgroup
        const bool points = ch.fused || (ch.tails && ch.C == 1);
        if (ch.fused) e = sig::trunc_backward_tails_fused(w.d, w.depth, path, coeffs, grad_coeffs, B, n_points, ch.C, ch.Lc, grad_path, st);
        else if (ch.tails)
            e = sig::trunc_backward_tails(w.d, w.depth, path, row_coeffs, row_grad, B, n_points, ch.C, ch.Lc, gdx,
                                          points ? grad_path : nullptr, st);
        else e = sig::trunc_backward(w.d, w.depth, path, row_coeffs, row_grad, nullptr, nullptr, B, n_points, ch.C, ch.Lc, gdx, residual,
                                     w.opt.bwd_tile, st);
        if (pe) (void)hipEventRecord(pe[1], st);
        if (e != hipSuccess) return hip_fail(e);
        if (!points) e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    if (use_lanes(w, B)) {
        const sig::LanesShape ls = lanes_shape_for(w, 1, B);
        g_not_ready = false;
        sig::JitKernel* lk = ensure_lanes(w, 1, ls, how);
        if (!lk && g_not_ready) return SIG_ENOTREADY;
        if (lk) {
            hipEvent_t* pe = g_prof.next(1);
            if (pe) (void)hipEventRecord(pe[0], st);
            e = launch_lanes(*lk, ls, path, coeffs, grad_coeffs, B, n_points, gdx, st);
            if (pe) (void)hipEventRecord(pe[1], st);
            if (e != hipSuccess) return hip_fail(e);
            e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    const sig::Plan* jp = nullptr;
    g_not_ready = false;
    sig::JitKernel* jk = ensure_jit(w, 1, B, how, &jp);
    if (!jk && g_not_ready) return SIG_ENOTREADY;
    if (jk) {
        // increment gradients and increments in the same layout [group][padded segment][letter][lane], one after the other
        const size_t t_bytes = jit_dxt_bytes(w, B, n_points, 1);
        const size_t gdx_bytes = std::max(gdx_bytes_of(w, B, n_points), t_bytes);
        float* dxT = (float*)((unsigned char*)workspace + gdx_bytes);
        const int64_t Lpad = jit_lpad(w, n_points, 1);
        e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, gdx, st);   // clears the gradients as well
        if (e != hipSuccess) return hip_fail(e);
        hipEvent_t* pe = g_prof.next(1);
        if (pe) (void)hipEventRecord(pe[0], st);
        e = launch_jit_backward(*jk, *jp, dxT, coeffs, grad_coeffs, B, n_points - 1, Lpad / jk->tile, w.size(),
                                gdx, st);
        if (pe) (void)hipEventRecord(pe[1], st);
        if (e != hipSuccess) return hip_fail(e);
        e = sig::grad_points_transposed(gdx, B, n_points, w.d, Lpad, grad_path, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    if (maybe_jit) {                     // no specialised kernel after all: the table-driven one takes gdx [B][L][d]
        e = sig::fill_zero(gdx, B * (n_points - 1) * w.d, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    const int v = pick_variant(w, 1, B);
    const sig::Plan& p = w.plans[1][(size_t)v];
    const auto& po = w.offsets[1][(size_t)v];
    const unsigned char* base = (const unsigned char*)w.dev;
    sig::GenericArgs a;
    a.units = (const sig::UnitDesc*)(base + po.units);
    a.ops = (const uint32_t*)(base + po.ops);
    a.slot_word = (const int32_t*)(base + po.slots);
    a.n_units = (int64_t)p.units.size();
    a.max_slots = p.max_slots;
    a.path = path; a.B = B; a.P = n_points; a.d = w.d; a.nW = w.size();
    a.coeffs_in = coeffs; a.grad_coeffs = grad_coeffs; a.gdx = gdx;
    a.tile_steps = bwd_tile_steps(w.d);
    hipEvent_t* pe = g_prof.next(1);
    if (pe) (void)hipEventRecord(pe[0], st);
    e = sig::generic_backward(a, w.max_len, st);
    if (pe) (void)hipEventRecord(pe[1], st);
    if (e != hipSuccess) return hip_fail(e);
    e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_backward(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                 int64_t n_points, float* grad_path, void* workspace, size_t workspace_bytes, void* stream)
{
    return backward_impl(ws, path, coeffs, grad_coeffs, B, n_points, grad_path, workspace, workspace_bytes, stream,
                         Build::compile_and_load);
}

size_t sig_checkpoint_bytes(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    if (!ws || B <= 0 || n_points <= 1) return 0;
    const Chunks ch = checkpoint_chunks(*W(ws), B, n_points);
    return ch.C >= 2 ? chunk_array_bytes(*W(ws), B, ch.C) : 0;
}

int64_t sig_checkpoint_chunks(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    if (!ws || B <= 0 || n_points <= 1) return 1;
    const Chunks ch = checkpoint_chunks(*W(ws), B, n_points);
    return ch.C >= 2 ? ch.C : 1;
}

size_t sig_forward_checkpointed_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    if (!ws || B <= 0 || n_points <= 1) return 0;
    const Chunks ch = checkpoint_chunks(*W(ws), B, n_points);
    if (ch.C < 2) return sig_forward_workspace_bytes(ws, B, n_points);
    if (W(ws)->kind != 0) return std::max(words_forward_ckpt_workspace(*W(ws), B, ch), jit_dxt_bytes(*W(ws), B, n_points, 0));
    return forward_chunk_arrays(*W(ws), ch.C) > 1 ? chunk_array_bytes(*W(ws), B, ch.C) : 0;   // partial products of four chunks
}

size_t sig_backward_checkpointed_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points)
{
    if (!ws || B <= 0 || n_points <= 1) return 0;
    const sig::WordSet& w = *W(ws);
    const Chunks ch = checkpoint_chunks(w, B, n_points);
    if (ch.C < 2) return sig_backward_workspace_bytes(ws, B, n_points);
    if (w.kind != 0) return std::max(words_backward_ckpt_workspace(w, B, ch), sig_backward_workspace_bytes(ws, B, n_points));
    // gradient of the increments, boundary adjoints; beyond two chunks also the products before and after every chunk
    return gdx_bytes_of(w, B, n_points) + chunk_array_bytes(w, B, ch.C - 1) + (ch.C == 2 ? 0 : 2) * chunk_array_bytes(w, B, ch.C);
}

int sig_forward_checkpointed(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, float* coeffs,
                             void* checkpoint, size_t checkpoint_bytes, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    const sig::WordSet& w = *W(ws);
    const Chunks ch = (B > 0 && n_points > 1) ? checkpoint_chunks(w, B, n_points) : Chunks{1, 0};
    if (ch.C < 2) return sig_forward(ws, path, B, n_points, coeffs, workspace, workspace_bytes, stream);
    if (!coeffs) return SIG_EINVAL;
    const size_t nb = chunk_array_bytes(w, B, ch.C);
    if (!checkpoint || checkpoint_bytes < nb) return SIG_EWORKSPACE;
    if (w.kind != 0) {
        if (((uintptr_t)checkpoint & 255) != 0) return SIG_EINVAL;
        sig::JitKernel *fk, *bk;
        const sig::Plan *fp = nullptr, *bp = nullptr;
        if (!words_kernels(w, B * ch.C, &fk, &fp, &bk, &bp))
            return forward_impl(ws, path, B, n_points, coeffs, workspace, workspace_bytes, stream, false);
        if (!workspace || workspace_bytes < sig_forward_checkpointed_workspace_bytes(ws, B, n_points)) return SIG_EWORKSPACE;
        if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
        hipStream_t st = (hipStream_t)stream;
        CallTimer whole(0, st);
        hipError_t e = words_forward_chunked(w, path, B, n_points, ch, *fk, *fp, (float*)workspace, (float*)checkpoint, coeffs, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    if (((uintptr_t)checkpoint & 255) != 0 || ((uintptr_t)coeffs & 15) != 0) return SIG_EINVAL;
    float* Pfx = nullptr;
    if (forward_chunk_arrays(w, ch.C) > 1) {
        if (!workspace || workspace_bytes < nb) return SIG_EWORKSPACE;
        if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
        Pfx = (float*)workspace;
    }
    hipStream_t st = (hipStream_t)stream;
    CallTimer whole(0, st);
    float* Sc = (float*)checkpoint;
    hipEvent_t* pe = g_prof.next(0);
    if (pe) (void)hipEventRecord(pe[0], st);
    hipError_t e = sig::trunc_forward(w.d, w.depth, path, B, n_points, ch.C, ch.Lc, Sc, st);
    if (pe) (void)hipEventRecord(pe[1], st);
    if (e == hipSuccess) e = sig::chunk_scan(w.d, w.depth, Sc, Pfx, nullptr, nullptr, coeffs, nullptr, nullptr, B, (int)ch.C, nullptr, st);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_backward_checkpointed(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs,
                              const void* checkpoint, size_t checkpoint_bytes, int64_t B, int64_t n_points, float* grad_path,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    const sig::WordSet& w = *W(ws);
    const Chunks ch = (B > 0 && n_points > 1) ? checkpoint_chunks(w, B, n_points) : Chunks{1, 0};
    if (ch.C < 2) return sig_backward(ws, path, coeffs, grad_coeffs, B, n_points, grad_path, workspace, workspace_bytes, stream);
    if (!coeffs || !grad_coeffs || !grad_path) return SIG_EINVAL;
    if (!checkpoint || checkpoint_bytes < chunk_array_bytes(w, B, ch.C)) return SIG_EWORKSPACE;
    if (w.kind != 0) {
        sig::JitKernel *fk, *bk;
        const sig::Plan *fp = nullptr, *bp = nullptr;
        if (!words_kernels(w, B * ch.C, &fk, &fp, &bk, &bp))
            return sig_backward(ws, path, coeffs, grad_coeffs, B, n_points, grad_path, workspace, workspace_bytes, stream);
        if (!workspace || workspace_bytes < sig_backward_checkpointed_workspace_bytes(ws, B, n_points)) return SIG_EWORKSPACE;
        if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)checkpoint & 255) != 0) return SIG_EINVAL;
        hipStream_t st = (hipStream_t)stream;
        CallTimer whole(1, st);
        hipError_t e = words_backward_chunked(w, path, coeffs, grad_coeffs, (const float*)checkpoint, ch, B, n_points, grad_path,
                                              workspace, *bk, *bp, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    if (!workspace || workspace_bytes < sig_backward_checkpointed_workspace_bytes(ws, B, n_points)) return SIG_EWORKSPACE;
    if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)checkpoint & 255) != 0) return SIG_EINVAL;
    return backward_checkpointed(w, path, coeffs, grad_coeffs, (const float*)checkpoint, ch, B, n_points, grad_path, workspace,
                                 (hipStream_t)stream);
}

int sig_backward_residual(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                          int64_t n_points, float* grad_path, float* residual, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    if (!residual) return SIG_EINVAL;
    if (ws && B > 0 && n_points == 1) {
        hipError_t e = sig::fill_zero(residual, B, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    return backward_impl(ws, path, coeffs, grad_coeffs, B, n_points, grad_path, workspace, workspace_bytes, stream,
                         Build::compile_and_load, residual);
}

int sig_backward_static(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                        int64_t n_points, float* grad_path, void* stream)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    if (backward_workspace(ws, B, n_points, false) > (size_t)SIG_STATIC_SCRATCH_BYTES) return SIG_ETOOLARGE;
    void* scratch_ptr = nullptr;                         // this device's copy of the static array
    hipError_t e = sig::static_scratch(&scratch_ptr);
    if (e != hipSuccess) return hip_fail(e);
    return backward_impl(ws, path, coeffs, grad_coeffs, B, n_points, grad_path, scratch_ptr, (size_t)SIG_STATIC_SCRATCH_BYTES, stream,
                         Build::loaded_only, nullptr, false);
}

// ---- windows: every (path, window) pair is gathered into a path of its own (padded with its last point), the
// ordinary forward / backward runs on those B * K paths, and the gradient is scattered back.
static size_t win_sub_bytes(const sig::WordSet& w, int64_t B, int64_t K, int64_t n_sub)
{
    return ((size_t)B * (size_t)K * (size_t)n_sub * (size_t)w.d * sizeof(float) + 255) & ~(size_t)255;
}

// Full truncations with register-resident kernels read every window straight from the path (no copy of the path per
// window, short windows end early); other word sets take the gather into padded sub-paths.
static bool windows_direct(const sig::WordSet& w, int64_t B, int64_t K, int backward)
{
    return B * K <= 65535 && (backward ? use_trunc_backward(w, B * K) : use_trunc_forward(w, B * K));
}
// Word sets that run through the straight-line specialised kernels (lane = row): their rows can be windows as well,
// the increments being transposed straight from the path.  (The workspace the window calls ask for covers both this
// form and the gather into padded sub-paths, which the other kernels and a failed compilation take.)
static bool windows_rows_jit(const sig::WordSet& w, int64_t rows)
{
    return !use_trunc_forward(w, rows) && !use_trunc_backward(w, rows) && !use_lanes(w, rows) && jit_enabled(w);
}

size_t sig_forward_windows_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points, int64_t K, int64_t max_window_len)
{
    if (!ws || B <= 0 || K <= 0 || n_points < 1 || max_window_len < 0) return 0;
    if (windows_direct(*W(ws), B, K, 0)) return 0;
    const int64_t n_sub = max_window_len + 1;
    return win_sub_bytes(*W(ws), B, K, n_sub) + sig_forward_workspace_bytes(ws, B * K, n_sub);
}

size_t sig_backward_windows_workspace_bytes(const sig_wordset* ws, int64_t B, int64_t n_points, int64_t K, int64_t max_window_len)
{
    if (!ws || B <= 0 || K <= 0 || n_points < 1 || max_window_len < 0) return 0;
    if (windows_direct(*W(ws), B, K, 1)) return n_points > 1 ? gdx_bytes_of(*W(ws), B, n_points) : 0;
    const int64_t n_sub = max_window_len + 1;
    // the gather form; the forms that take windows as rows need less, or (a word per lane) the increment gradients of
    // the whole paths
    const size_t gather = 2 * win_sub_bytes(*W(ws), B, K, n_sub) + sig_backward_workspace_bytes(ws, B * K, n_sub);
    return n_points > 1 ? std::max(gather, gdx_bytes_of(*W(ws), B, n_points)) : gather;
}

int sig_forward_windows(const sig_wordset* ws, const float* path, int64_t B, int64_t n_points, const int64_t* windows, int64_t K,
                        int64_t max_window_len, float* coeffs, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    if (K < 0 || max_window_len < 0 || max_window_len > n_points - 1) return SIG_EINVAL;
    if (B == 0 || K == 0) return SIG_OK;
    if (!windows || !coeffs) return SIG_EINVAL;
    if (B * K > (int64_t)65535 * 64) return SIG_ETOOLARGE;
    const sig::WordSet& w = *W(ws);
    if (windows_direct(w, B, K, 0)) {
        hipStream_t st = (hipStream_t)stream;
        if (n_points == 1 || max_window_len == 0) {
            hipError_t e0 = sig::fill_zero(coeffs, B * K * w.size(), st);
            return e0 == hipSuccess ? SIG_OK : hip_fail(e0);
        }
        CallTimer whole(0, st);
        sig::WindowList wl;
        wl.win = windows; wl.K = K; wl.max_len = max_window_len;
        hipEvent_t* pe = g_prof.next(0);
        if (pe) (void)hipEventRecord(pe[0], st);
        hipError_t e1 = sig::trunc_forward_windows(w.d, w.depth, path, B, n_points, wl, coeffs, st);
        if (pe) (void)hipEventRecord(pe[1], st);
        return e1 == hipSuccess ? SIG_OK : hip_fail(e1);
    }
    const int64_t n_sub = max_window_len + 1;
    const size_t sb = win_sub_bytes(w, B, K, n_sub);
    if (!workspace || workspace_bytes < sig_forward_windows_workspace_bytes(ws, B, n_points, K, max_window_len)) return SIG_EWORKSPACE;
    if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
    // a word per lane (full truncations of any alphabet size): every (path, window) row reads its window of the path
    if (!use_trunc_forward(w, B * K) && use_lanes(w, B * K) && n_points > 1 && max_window_len > 0) {
        const sig::LanesShape ls = lanes_shape_for(w, 0, B * K);
        if (sig::JitKernel* lk = ensure_lanes(w, 0, ls, Build::compile_and_load)) {
            hipStream_t st = (hipStream_t)stream;
            CallTimer whole(0, st);
            sig::WindowList wl;
            wl.win = windows; wl.K = K; wl.max_len = max_window_len;
            hipEvent_t* pe = g_prof.next(0);
            if (pe) (void)hipEventRecord(pe[0], st);
            hipError_t e = launch_lanes(*lk, ls, path, nullptr, nullptr, B, n_points, coeffs, st, wl);
            if (pe) (void)hipEventRecord(pe[1], st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    // straight-line specialised kernels: the rows' increments are transposed straight from the path, window by window
    if (windows_rows_jit(w, B * K) && n_points > 1 && max_window_len > 0) {
        const sig::Plan* jp = nullptr;
        if (sig::JitKernel* jk = ensure_jit(w, 0, B * K, Build::compile_and_load, &jp)) {
            hipStream_t st = (hipStream_t)stream;
            CallTimer whole(0, st);
            sig::WindowList wl;
            wl.win = windows; wl.K = K; wl.max_len = max_window_len;
            float* dxT = (float*)workspace;
            const int64_t Lpad = jit_lpad(w, n_sub, 0);
            hipError_t e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, nullptr, st, wl);
            if (e != hipSuccess) return hip_fail(e);
            hipEvent_t* pe = g_prof.next(0);
            if (pe) (void)hipEventRecord(pe[0], st);
            e = launch_jit_forward(*jk, *jp, dxT, B * K, Lpad / jk->tile, coeffs, w.size(), st);
            if (pe) (void)hipEventRecord(pe[1], st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    float* sub = (float*)workspace;
    hipError_t e = sig::window_gather(path, B, n_points, w.d, windows, K, n_sub, sub, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
    return sig_forward(ws, sub, B * K, n_sub, coeffs, (unsigned char*)workspace + sb, workspace_bytes - sb, stream);
}

int sig_backward_windows(const sig_wordset* ws, const float* path, const float* coeffs, const float* grad_coeffs, int64_t B,
                         int64_t n_points, const int64_t* windows, int64_t K, int64_t max_window_len, float* grad_path,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_common(ws, path, B, n_points);
    if (rc != SIG_OK) return rc;
    if (K < 0 || max_window_len < 0 || max_window_len > n_points - 1) return SIG_EINVAL;
    if (B == 0) return SIG_OK;
    if (!grad_path) return SIG_EINVAL;
    const sig::WordSet& w = *W(ws);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = sig::fill_zero(grad_path, B * n_points * w.d, st);
    if (e != hipSuccess) return hip_fail(e);
    if (K == 0) return SIG_OK;
    if (!windows || !coeffs || !grad_coeffs) return SIG_EINVAL;
    if (B * K > (int64_t)65535 * 64) return SIG_ETOOLARGE;
    if (windows_direct(w, B, K, 1)) {
        if (n_points == 1 || max_window_len == 0) return SIG_OK;            // grad_path is zero already
        if (!workspace || workspace_bytes < gdx_bytes_of(w, B, n_points)) return SIG_EWORKSPACE;
        if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
        CallTimer whole(1, st);
        float* gdx = (float*)workspace;
        e = sig::fill_zero(gdx, B * (n_points - 1) * w.d, st);
        if (e != hipSuccess) return hip_fail(e);
        sig::WindowList wl;
        wl.win = windows; wl.K = K; wl.max_len = max_window_len;
        hipEvent_t* pe = g_prof.next(1);
        if (pe) (void)hipEventRecord(pe[0], st);
        e = sig::trunc_backward_windows(w.d, w.depth, path, coeffs, grad_coeffs, B, n_points, wl, gdx, st);
        if (pe) (void)hipEventRecord(pe[1], st);
        if (e != hipSuccess) return hip_fail(e);
        e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
        return e == hipSuccess ? SIG_OK : hip_fail(e);
    }
    const int64_t n_sub = max_window_len + 1;
    const size_t sb = win_sub_bytes(w, B, K, n_sub);
    if (!workspace || workspace_bytes < sig_backward_windows_workspace_bytes(ws, B, n_points, K, max_window_len)) return SIG_EWORKSPACE;
    if (((uintptr_t)workspace & 255) != 0) return SIG_EINVAL;
    // a word per lane: rows = windows read straight from the path, their increment gradients added up in gdx [B][L][d]
    // (at the start of the workspace, which is larger than that)
    if (!use_trunc_backward(w, B * K) && use_lanes(w, B * K) && n_points > 1 && max_window_len > 0 &&
        workspace_bytes >= gdx_bytes_of(w, B, n_points)) {
        const sig::LanesShape ls = lanes_shape_for(w, 1, B * K);
        if (sig::JitKernel* lk = ensure_lanes(w, 1, ls, Build::compile_and_load)) {
            CallTimer whole(1, st);
            sig::WindowList wl;
            wl.win = windows; wl.K = K; wl.max_len = max_window_len;
            float* gdx = (float*)workspace;
            e = sig::fill_zero(gdx, B * (n_points - 1) * w.d, st);
            if (e != hipSuccess) return hip_fail(e);
            hipEvent_t* pe = g_prof.next(1);
            if (pe) (void)hipEventRecord(pe[0], st);
            e = launch_lanes(*lk, ls, path, coeffs, grad_coeffs, B, n_points, gdx, st, wl);
            if (pe) (void)hipEventRecord(pe[1], st);
            if (e != hipSuccess) return hip_fail(e);
            e = sig::grad_points(gdx, B, n_points, w.d, grad_path, st);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    // straight-line specialised kernels: rows = windows, increments and their gradients in the transposed layout, the
    // chain rule adds every window's gradient into grad_path (needs 2 arrays of the transposed layout: less than asked)
    if (windows_rows_jit(w, B * K) && n_points > 1 && max_window_len > 0) {
        const sig::Plan* jp = nullptr;
        if (sig::JitKernel* jk = ensure_jit(w, 1, B * K, Build::compile_and_load, &jp)) {
            CallTimer whole(1, st);
            sig::WindowList wl;
            wl.win = windows; wl.K = K; wl.max_len = max_window_len;
            const size_t t_bytes = jit_dxt_bytes(w, B * K, n_sub, 1);
            float* gdx = (float*)workspace;
            float* dxT = (float*)((unsigned char*)workspace + t_bytes);
            const int64_t Lpad = jit_lpad(w, n_sub, 1);
            e = sig::increments_transposed(path, B, n_points, w.d, Lpad, dxT, gdx, st, wl);
            if (e != hipSuccess) return hip_fail(e);
            hipEvent_t* pe = g_prof.next(1);
            if (pe) (void)hipEventRecord(pe[0], st);
            e = launch_jit_backward(*jk, *jp, dxT, coeffs, grad_coeffs, B * K, max_window_len, Lpad / jk->tile, w.size(), gdx, st);
            if (pe) (void)hipEventRecord(pe[1], st);
            if (e != hipSuccess) return hip_fail(e);
            e = sig::grad_points_transposed(gdx, B, n_points, w.d, Lpad, grad_path, st, wl);
            return e == hipSuccess ? SIG_OK : hip_fail(e);
        }
    }
    float* sub = (float*)workspace;
    float* gsub = (float*)((unsigned char*)workspace + sb);
    e = sig::window_gather(path, B, n_points, w.d, windows, K, n_sub, sub, st);
    if (e != hipSuccess) return hip_fail(e);
    rc = sig_backward(ws, sub, coeffs, grad_coeffs, B * K, n_sub, gsub, (unsigned char*)workspace + 2 * sb, workspace_bytes - 2 * sb,
                      stream);
    if (rc != SIG_OK) return rc;
    e = sig::window_scatter(gsub, B, n_points, w.d, windows, K, n_sub, grad_path, st);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_profile_enable(int on)
{
    g_prof.mask = on == 1 ? 0xFu : ((unsigned)on >> 1) & 0xFu;
    for (size_t& u : g_prof.used) u = 0;
    return SIG_OK;
}

int sig_profile_read(int which, int64_t* n_launches, double* total_ms)
{
    if (which < 0 || which > 3) return SIG_EINVAL;
    const int dir = which;
    double sum = 0.0;
    for (size_t k = 0; k < g_prof.used[dir]; ++k) {
        hipError_t e = hipEventSynchronize(g_prof.ev[dir][2 * k + 1]);
        if (e != hipSuccess) return hip_fail(e);
        float ms = 0.0f;
        e = hipEventElapsedTime(&ms, g_prof.ev[dir][2 * k], g_prof.ev[dir][2 * k + 1]);
        if (e != hipSuccess) return hip_fail(e);
        sum += ms;
    }
    if (n_launches) *n_launches = (int64_t)g_prof.used[dir];
    if (total_ms) *total_ms = sum;
    return SIG_OK;
}

const char* sig_strerror(int code)
{
    switch (code) {
        case SIG_OK: return "success";
        case SIG_EINVAL: return "invalid argument";
        case SIG_ELETTER: return "letter outside [0, d)";
        case SIG_EEMPTYWORD: return "empty word or empty word list";
        case SIG_ENOMEM: return "out of host memory";
        case SIG_EWORKSPACE: return "workspace or table buffer missing or too small";
        case SIG_EHIP: return "HIP runtime error";
        case SIG_ETOOLARGE: return "word set exceeds a format limit";
        case SIG_ENOTUPLOADED: return "word set tables not uploaded";
        case SIG_EUNSUPPORTED: return "not supported for this word set";
        case SIG_EJIT: return "run-time compilation failed";
        case SIG_ENOTREADY: return "the kernel for this word set and batch is not loaded yet (call sig_backward once first)";
        default: return "unknown error";
    }
}

int sig_last_hip_error(void) { return g_last_hip; }
const char* sig_version(void) { return "sig-mi355x 0.1"; }

const char* sig_wordset_kernel_name(const sig_wordset* ws, int backward)
{
    if (!ws || !W(ws)->kernels_supported) return "unsupported";
    if (!backward && use_trunc_forward(*W(ws), 1)) return "trunc_mfma_fwd_kernel";
    if (backward && use_trunc_backward(*W(ws), 1)) return sig::trunc_backward_kernel_name(W(ws)->d, W(ws)->depth);
    if (use_lanes(*W(ws), 1)) return backward ? "sig_bwd_lanes" : "sig_fwd_lanes";
    if (jit_enabled(*W(ws))) return backward ? "sig_bwd_jit" : "sig_fwd_jit";
    return backward ? "bwd_generic_kernel" : "fwd_generic_kernel";
}

int sig_jit_launch_shape_ok(int waves, int max_threads_per_block, int static_lds_bytes, int registers)
{
    return sig::jit_launch_shape_fits(waves, max_threads_per_block, static_lds_bytes, registers) ? 1 : 0;
}

int sig_probe_fma(void* out, size_t out_bytes, int blocks, int iters, void* stream)
{
    if (!out || blocks < 1 || iters < 1) return SIG_EINVAL;
    if (out_bytes < (size_t)blocks * 256 * sizeof(float)) return SIG_EWORKSPACE;
    hipError_t e = sig::fma_probe((float*)out, blocks, iters, (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

int sig_probe_issue(void* out, size_t out_bytes, int blocks, int iters, int mode, void* stream)
{
    if (!out || blocks < 1 || iters < 1 || mode < 0 || mode > 7) return SIG_EINVAL;
    if (out_bytes < (size_t)blocks * 256 * sizeof(float)) return SIG_EWORKSPACE;
    hipError_t e = sig::issue_probe((float*)out, blocks, iters, mode, (hipStream_t)stream);
    return e == hipSuccess ? SIG_OK : hip_fail(e);
}

const char* sig_kernel_name(const sig_wordset* ws, int backward, int64_t B, int64_t n_points)
{
    if (!ws || !W(ws)->kernels_supported) return "unsupported";
    const sig::WordSet& w = *W(ws);
    if (B < 1 || n_points < 2) return sig_wordset_kernel_name(ws, backward);
    if (!backward && use_trunc_forward(w, B))
        return trunc_forward_fused_chunks(w, B, n_points, nullptr) ? "trunc_tails_fwd_kernel" : "trunc_mfma_fwd_kernel";
    if (backward && use_trunc_backward(w, B)) {
        const BwdShape sh = trunc_backward_shape(w, B, n_points);
        return sh.tails ? "trunc_tails_bwd_kernel" : sig::trunc_backward_kernel_name(w.d, w.depth);
    }
    if (use_lanes(w, B)) return backward ? "sig_bwd_lanes" : "sig_fwd_lanes";
    if (jit_enabled(w)) return backward ? "sig_bwd_jit" : "sig_fwd_jit";
    return backward ? "bwd_generic_kernel" : "fwd_generic_kernel";
}

}  // extern "C"
