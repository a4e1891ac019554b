// Run-time specialisation of the signature kernels for one word set.
//
// For an arbitrary prefix-closed set the shape of the word tree is data.  Instead of interpreting the
// work-unit programs (kernels_generic.hip), this file prints each unit's program as straight-line HIP
// source - one multiply-add per (word, target length) pair, every coefficient a named register - and
// compiles it with hiprtc for gfx950.  Mapping as in the interpreter: one wavefront = one work unit x 64
// paths, lane = path; NW units of the same 64 paths share a workgroup and one LDS tile of increments.
//
// Forward step of a word u of length k (Algorithm 1 with shared intermediates), A_0 = 1:
//     A_k[t] = S(u) + dX^{(u_k)}/(t+1) * A_{k-1}[t+1],  t = 1..h(u);      S(u) += dX^{(u_k)} * A_{k-1}[1]
// Backward step (Section 4): reconstruction with -dX (Proposition 4.6), recompute with +dX, adjoint recursion
// (Proposition 4.1 with the right factors aggregated per prefix); see kernels_generic.hip for the formulas.
#include "jit.hpp"

#include <hip/hiprtc.h>
#include <unistd.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <set>
#include <sstream>
#include <utility>
#include <vector>

namespace sig {

namespace {

struct Op {
    int letter, level, h, kind;
};
inline Op decode(uint32_t w) { return Op{(int)(w & 0xfff), (int)((w >> 12) & 0xf), (int)((w >> 16) & 0xf), (int)((w >> 20) & 3)}; }

std::string fl(double v)
{
    char buf[64];
    std::snprintf(buf, sizeof buf, "%.9gf", v);
    std::string s(buf);
    if (s.find('.') == std::string::npos && s.find('e') == std::string::npos) s.insert(s.size() - 1, ".0");
    return s;
}

// name of dX^{(i)} / (t + 1)
std::string dxn(int i, int t) { return t == 0 ? "dx" + std::to_string(i) : "dx" + std::to_string(i) + "_" + std::to_string(t); }

void emit_prelude(std::ostringstream& o, int D, int T, int NW, bool backward)
{
    o << "#define D " << D << "\n#define T " << T << "\n#define NW " << NW << "\n";
    o << "#define TILE_F4 (T * D * 16)\n";                         // float4 per tile (T * D rows of 64 floats)
    o << "#define EPT ((TILE_F4 + NW * 64 - 1) / (NW * 64))\n";    // float4 per thread
    o << R"SRC(
typedef float f4 __attribute__((ext_vector_type(4)));
// The increments arrive differenced and transposed (increments_transposed_kernel): for the 64 paths of the
// workgroup, dxg[(j * D + i) * 64 + lane], zero for segments j >= L, and the segment count padded to a multiple
// of T, so a tile is one contiguous block that the workgroup copies to LDS with 16-byte accesses.
__device__ __forceinline__ void tile_fetch(const float* __restrict__ dxg, long tile_idx, int tid, f4 (&r)[EPT])
{
    const f4* p = (const f4*)dxg + (tile_idx < 0 ? 0 : tile_idx) * TILE_F4;
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int e = tid + q * NW * 64;
        r[q] = p[e < TILE_F4 ? e : TILE_F4 - 1];
    }
}
__device__ __forceinline__ void tile_stage(float* tile, int tid, const f4 (&r)[EPT])
{
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int e = tid + q * NW * 64;
        if (e < TILE_F4) ((f4*)tile)[e] = r[q];
    }
}
)SRC";
    if (!backward) {
        o << R"SRC(
// a wavefront without a unit still takes part in loading the tiles and in the barriers
__device__ __attribute__((noinline)) void idle_unit(const float* __restrict__ dxg, long ntiles, float* tile, int tid)
{
    f4 r[EPT];
    tile_fetch(dxg, 0, tid, r);
    tile_stage(tile, tid, r);
    __syncthreads();
    for (long n = 0; n < ntiles; ++n) {
        tile_fetch(dxg, n + 1 < ntiles ? n + 1 : n, tid, r);
        __syncthreads();
        tile_stage(tile, tid, r);
        __syncthreads();
    }
}
)SRC";
    } else {
        o << R"SRC(
// Gradient tiles: every wavefront (unit) has its own gt[(tt * D + i) * 64 + lane] in LDS and overwrites all of it
// in every tile with plain stores (LDS floating-point atomics turned out to be far slower than the arithmetic).
// At the end of a tile the NW tiles are added up and added to the increment gradients, which the specialised kernels
// keep in the layout of the increments themselves, gdx[group][segment][letter][lane] (zeroed by the caller): a row of
// a tile is 64 consecutive floats, one floating-point atomic instruction of full cache lines; all workgroup columns
// (blockIdx.x) add into the same array.
#define GT_F (T * D * 64)
__device__ __attribute__((noinline)) void grad_flush(const float* gt_all, float* gdx_tile, int lane, int wib)
{
    for (int e = wib; e < T * D; e += NW) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += gt_all[w * GT_F + e * 64 + lane];
        __hip_atomic_fetch_add(gdx_tile + e * 64 + lane, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
__device__ __attribute__((noinline)) void idle_unit(const float* __restrict__ dxg, long ntiles, long L, float* tile, float* gt_all,
                                                    float* gdx, long b0, long B, int lane, int wib)
{
    f4 r[EPT];
    const int tid = wib * 64 + lane;
    float* gt = gt_all + wib * GT_F;
    for (int e = lane; e < GT_F; e += 64) gt[e] = 0.0f;       // this wavefront contributes nothing
    tile_fetch(dxg, ntiles - 1, tid, r);
    for (long n = ntiles - 1; n >= 0; --n) {
        __syncthreads();
        tile_stage(tile, tid, r);
        __syncthreads();
        tile_fetch(dxg, n - 1, tid, r);
        __syncthreads();
        grad_flush(gt_all, gdx + n * (long)(T * D * 64), lane, wib);
    }
}
)SRC";
    }
}

// letters and scaled copies a unit uses
struct Uses {
    std::set<int> letters;
    std::set<std::pair<int, int>> scaled;   // (letter, t >= 1)
};

Uses collect_uses(const Plan& plan, const UnitDesc& ud)
{
    Uses u;
    for (int q = 0; q < ud.n_ops; ++q) {
        const Op op = decode(plan.ops[(size_t)(ud.op_off + q)]);
        if (op.kind == OP_LEAVE) continue;
        u.letters.insert(op.letter);
        for (int t = 1; t <= op.h; ++t) u.scaled.insert({op.letter, t});
    }
    return u;
}

void emit_step_loads(std::ostringstream& o, const Uses& u, const char* indent)
{
    for (int i : u.letters) o << indent << "const float dx" << i << " = dxp[" << i * 64 << "];\n";
    for (auto& it : u.scaled)
        o << indent << "const float " << dxn(it.first, it.second) << " = dx" << it.first << " * " << fl(1.0 / (it.second + 1)) << ";\n";
}

void emit_forward_unit(std::ostringstream& o, const Plan& plan, int uidx)
{
    const UnitDesc& ud = plan.units[(size_t)uidx];
    const Uses uses = collect_uses(plan, ud);
    o << "__device__ __forceinline__ void fwd_unit_" << uidx
      << "(const float* __restrict__ dxg, long ntiles, float* tile, int lane, int wib, float* __restrict__ out)\n{\n";
    o << "    float";
    for (int r = 0; r < ud.n_slots; ++r) o << (r ? ", " : " ") << "s" << r << " = 0.0f";
    o << ";\n";
    o << "    const int tid = wib * 64 + lane;\n";
    o << "    f4 r[EPT];\n    tile_fetch(dxg, 0, tid, r);\n    tile_stage(tile, tid, r);\n    __syncthreads();\n";
    o << "    for (long n = 0; n < ntiles; ++n) {\n";
    o << "        tile_fetch(dxg, n + 1 < ntiles ? n + 1 : n, tid, r);\n";
    // the segment loop is unrolled by two only: the loop bodies of all resident units together must fit the
    // instruction cache
    o << "#pragma unroll 2\n        for (int tt = 0; tt < T; ++tt) {\n";
    o << "            const float* dxp = tile + tt * D * 64 + lane;\n";
    emit_step_loads(o, uses, "            ");
    int depth = 0;   // open scopes = length of the current word chain
    int slot = 0;
    for (int q = 0; q < ud.n_ops; ++q) {
        const Op op = decode(plan.ops[(size_t)(ud.op_off + q)]);
        while (depth >= op.level) { o << "            }\n"; --depth; }
        o << "            {\n";
        ++depth;
        const std::string s = "s" + std::to_string(slot);
        const int k = op.level;
        for (int t = 1; t <= op.h; ++t) {
            o << "                const float a" << k << "_" << t << " = ";
            if (k == 1) o << s << " + " << dxn(op.letter, t) << ";\n";
            else o << "__builtin_fmaf(" << dxn(op.letter, t) << ", a" << k - 1 << "_" << t + 1 << ", " << s << ");\n";
        }
        if (k == 1) o << "                " << s << " += dx" << op.letter << ";\n";
        else o << "                " << s << " = __builtin_fmaf(dx" << op.letter << ", a" << k - 1 << "_1, " << s << ");\n";
        ++slot;
    }
    while (depth > 0) { o << "            }\n"; --depth; }
    o << "        }\n        __syncthreads();\n        tile_stage(tile, tid, r);\n        __syncthreads();\n    }\n";
    o << "    if (out) {\n";
    for (int r = 0; r < ud.n_slots; ++r) {
        const int32_t w = plan.slot_word[(size_t)(ud.slot_off + r)];
        if (w >= 0) o << "        out[" << w << "] = s" << r << ";\n";
    }
    o << "    }\n}\n\n";
}

void emit_backward_unit(std::ostringstream& o, const Plan& plan, int uidx, int D_of_plan)
{
    const UnitDesc& ud = plan.units[(size_t)uidx];
    const Uses uses = collect_uses(plan, ud);
    o << "__device__ __forceinline__ void bwd_unit_" << uidx
      << "(const float* __restrict__ dxg, long ntiles, long L, float* tile, float* gt_all, float* gdx, long b0, long B, int lane,\n"
         "     int wib, const float* __restrict__ cf, const float* __restrict__ gr)\n{\n";
    // slots of words with children carry a coefficient; the others only an adjoint
    std::vector<char> has_children((size_t)ud.n_slots, 0);
    for (int q = 0, slot = 0; q < ud.n_ops; ++q) {
        const Op op = decode(plan.ops[(size_t)(ud.op_off + q)]);
        if (op.kind == OP_ENTER) has_children[(size_t)slot++] = 1;
        else if (op.kind == OP_LEAF) ++slot;
    }
    for (int r = 0; r < ud.n_slots; ++r) {
        const int32_t w = plan.slot_word[(size_t)(ud.slot_off + r)];
        const int32_t wi = w >= 0 ? w : ~w;
        o << "    float ";
        if (has_children[(size_t)r]) o << "s" << r << " = cf[" << wi << "], ";
        o << "ab" << r << " = ";
        if (w >= 0) o << "gr[" << wi << "];\n";
        else o << "0.0f;\n";
    }
    o << "    const int tid = wib * 64 + lane;\n";
    o << "    f4 r[EPT];\n    float* gt = gt_all + wib * GT_F;\n";
    o << "    tile_fetch(dxg, ntiles - 1, tid, r);\n";
    o << "    for (long n = ntiles - 1; n >= 0; --n) {\n";
    o << "        __syncthreads();\n        tile_stage(tile, tid, r);\n        __syncthreads();\n";
    o << "        tile_fetch(dxg, n - 1, tid, r);\n";
    // not unrolled: measured as fast as unrolled by two, and the compilation is a quarter shorter
    o << "#pragma unroll 1\n        for (int tt = T - 1; tt >= 0; --tt) {\n";
    o << "            const float* dxp = tile + tt * D * 64 + lane;\n";
    emit_step_loads(o, uses, "            ");
    for (int i : uses.letters) o << "            float g" << i << " = 0.0f;\n";
    int slot = 0;
    std::vector<int> open_slot(16, 0);
    for (int q = 0; q < ud.n_ops; ++q) {
        const Op op = decode(plan.ops[(size_t)(ud.op_off + q)]);
        const int k = op.level, i = op.letter;
        const std::string ind = "                ";
        if (op.kind == OP_ENTER) {
            const std::string s = "s" + std::to_string(slot);
            open_slot[(size_t)k] = slot;
            o << "            {\n";
            for (int t = 1; t <= op.h; ++t) {
                o << ind << "const float m" << k << "_" << t << " = ";
                if (k == 1) o << s << " - " << dxn(i, t) << ";\n";
                else o << "__builtin_fmaf(-" << dxn(i, t) << ", m" << k - 1 << "_" << t + 1 << ", " << s << ");\n";
            }
            if (k == 1) o << ind << s << " -= dx" << i << ";\n";
            else o << ind << s << " = __builtin_fmaf(-dx" << i << ", m" << k - 1 << "_1, " << s << ");\n";
            for (int t = 1; t <= op.h; ++t) {
                o << ind << "const float p" << k << "_" << t << " = ";
                if (k == 1) o << s << " + " << dxn(i, t) << ";\n";
                else o << "__builtin_fmaf(" << dxn(i, t) << ", p" << k - 1 << "_" << t + 1 << ", " << s << ");\n";
            }
            o << ind << "float";
            for (int t = 1; t <= op.h; ++t) o << (t > 1 ? ", " : " ") << "q" << k << "_" << t << " = 0.0f";
            o << ";\n";
            ++slot;
        } else if (op.kind == OP_LEAF) {
            const std::string s = "s" + std::to_string(slot), b = "ab" + std::to_string(slot);
            // the coefficient of a word without children is not reconstructed: nothing reads it
            if (k == 1) {
                o << "            g" << i << " += " << b << ";\n";
            } else {
                o << "            g" << i << " = __builtin_fmaf(" << b << ", p" << k - 1 << "_1, g" << i << ");\n";
                o << "            q" << k - 1 << "_1 = __builtin_fmaf(dx" << i << ", " << b << ", q" << k - 1 << "_1);\n";
            }
            ++slot;
        } else {   // LEAVE
            const std::string b = "ab" + std::to_string(open_slot[(size_t)k]);
            if (k == 1) {
                o << ind << "g" << i << " += " << b << ";\n";
                for (int t = 1; t <= op.h; ++t) o << ind << "g" << i << " = __builtin_fmaf(q1_" << t << ", " << fl(1.0 / (t + 1)) << ", g" << i << ");\n";
            } else {
                o << ind << "g" << i << " = __builtin_fmaf(" << b << ", p" << k - 1 << "_1, g" << i << ");\n";
                o << ind << "q" << k - 1 << "_1 = __builtin_fmaf(dx" << i << ", " << b << ", q" << k - 1 << "_1);\n";
                for (int t = 1; t <= op.h; ++t) {
                    o << ind << "g" << i << " = __builtin_fmaf(q" << k << "_" << t << " * " << fl(1.0 / (t + 1)) << ", p" << k - 1 << "_" << t + 1
                      << ", g" << i << ");\n";
                    o << ind << "q" << k - 1 << "_" << t + 1 << " = __builtin_fmaf(" << dxn(i, t) << ", q" << k << "_" << t << ", q" << k - 1 << "_"
                      << t + 1 << ");\n";
                }
            }
            o << ind << b << " = " << b;
            for (int t = 1; t <= op.h; ++t) o << " + q" << k << "_" << t;
            o << ";\n";
            o << "            }\n";
        }
    }
    o << "            float* gp = gt + tt * D * 64 + lane;\n";
    for (int i = 0; i < D_of_plan; ++i) {
        if (uses.letters.count(i)) o << "            gp[" << i << " * 64] = g" << i << ";\n";
        else o << "            gp[" << i << " * 64] = 0.0f;\n";
    }
    o << "        }\n";
    o << "        __syncthreads();\n        grad_flush(gt_all, gdx + n * (long)(T * D * 64), lane, wib);\n    }\n}\n\n";
}

}  // namespace

std::string jit_forward_source(const WordSet& ws, const Plan& plan, int NW, int T)
{
    std::ostringstream o;
    emit_prelude(o, ws.d, T, NW, false);
    const int nu = (int)plan.units.size();
    for (int u = 0; u < nu; ++u) emit_forward_unit(o, plan, u);
    o << "extern \"C\" __global__ __launch_bounds__(NW * 64) void sig_fwd_jit(const float* __restrict__ dxT, long B, long ntiles,\n"
         "                                                                  float* __restrict__ coeffs, long nW)\n{\n";
    o << "    __shared__ __attribute__((aligned(16))) float tile[T * D * 64];\n";
    o << "    const int lane = threadIdx.x & 63;\n    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
    o << "    const long b = (long)blockIdx.y * 64 + lane;\n    const bool valid = b < B;\n";
    o << "    const float* dxg = dxT + (long)blockIdx.y * ntiles * (T * D * 64);\n";
    o << "    float* out = valid ? coeffs + b * nW : nullptr;\n";
    o << "    const int unit = blockIdx.x * NW + wib;\n    switch (unit) {\n";
    for (int u = 0; u < nu; ++u) o << "        case " << u << ": fwd_unit_" << u << "(dxg, ntiles, tile, lane, wib, out); break;\n";
    o << "        default: idle_unit(dxg, ntiles, tile, wib * 64 + lane); break;\n    }\n}\n";
    return o.str();
}

std::string jit_backward_source(const WordSet& ws, const Plan& plan, int NW, int T)
{
    std::ostringstream o;
    emit_prelude(o, ws.d, T, NW, true);
    const int nu = (int)plan.units.size();
    for (int u = 0; u < nu; ++u) emit_backward_unit(o, plan, u, ws.d);
    o << "extern \"C\" __global__ __launch_bounds__(NW * 64) void sig_bwd_jit(const float* __restrict__ dxT,\n"
         "        const float* __restrict__ coeffs, const float* __restrict__ grad, long B, long L, long ntiles, long nW, float* gdx,\n"
         "        const float* __restrict__ coeffs_last, const float* __restrict__ grad_last, long C)\n{\n";
    o << "    __shared__ __attribute__((aligned(16))) float tile[T * D * 64];\n    __shared__ float gt[NW * GT_F];\n";
    o << "    const int lane = threadIdx.x & 63;\n    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
    o << "    const long b0 = (long)blockIdx.y * 64;\n    const long b = b0 + lane;\n    const long bc = b < B ? b : B - 1;\n";
    o << "    const float* dxg = dxT + (long)blockIdx.y * ntiles * (T * D * 64);\n";
    o << "    gdx += (long)blockIdx.y * ntiles * (T * D * 64);\n";
    // rows are the C time chunks of B / C paths: the last chunk of a path starts from the terminal signature and the
    // gradient themselves (arrays of one row per path), the others from rows of the per-chunk arrays; C = 1: whole paths
    o << "    const long pb = bc / C;\n    const bool last = bc - pb * C == C - 1;\n";
    o << "    const float* cf = last ? coeffs_last + pb * nW : coeffs + bc * nW;\n";
    o << "    const float* gr = last ? grad_last + pb * nW : grad + bc * nW;\n";
    o << "    const int unit = blockIdx.x * NW + wib;\n    switch (unit) {\n";
    for (int u = 0; u < nu; ++u)
        o << "        case " << u << ": bwd_unit_" << u << "(dxg, ntiles, L, tile, gt, gdx, b0, B, lane, wib, cf, gr); break;\n";
    o << "        default: idle_unit(dxg, ntiles, L, tile, gt, gdx, b0, B, lane, wib); break;\n    }\n}\n";
    return o.str();
}

namespace {
// Optional cache of compiled code objects on disk: with SIG_JIT_CACHE set to a directory, a code object is stored
// there under a 64-bit hash of its source (which carries every specialisation), the compiler version and the compile
// options, and later processes load it instead of compiling.  Files are written under a temporary name and renamed, so
// concurrent writers cannot leave a torn file; a file that fails its checks or does not load is removed and the
// kernel compiled afresh.
// the option list of every compilation; it enters the file name hash of the disk cache
const char* const kCompileOptions[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-munsafe-fp-atomics", "-Xclang", "-target-feature",
                                       "-Xclang", "-packed-fp32-ops"};
constexpr int kNumCompileOptions = (int)(sizeof kCompileOptions / sizeof kCompileOptions[0]);

uint64_t fnv1a(const char* p, size_t n, uint64_t h = 1469598103934665603ull)
{
    for (size_t i = 0; i < n; ++i) { h ^= (unsigned char)p[i]; h *= 1099511628211ull; }
    return h;
}
std::string cache_file(const std::string& src)
{
    const char* dir = std::getenv("SIG_JIT_CACHE");       // read when a kernel is compiled, never on the launch path
    if (!dir || !dir[0]) return std::string();
    int major = 0, minor = 0;
    (void)hiprtcVersion(&major, &minor);
    uint64_t h = fnv1a((const char*)&major, sizeof major);
    h = fnv1a((const char*)&minor, sizeof minor, h);
    for (const char* o : kCompileOptions) h = fnv1a(o, std::strlen(o) + 1, h);
    h = fnv1a(src.data(), src.size(), h);
    char name[64];
    std::snprintf(name, sizeof name, "/sig_gfx950_%016llx.hsaco", (unsigned long long)h);
    return std::string(dir) + name;
}
// File layout: 8 bytes magic, 8 bytes length of the code object, 8 bytes FNV-1a hash of it, then the code object.  A file
// that is short, foreign or damaged is not used.
constexpr char kCacheMagic[8] = {'S', 'I', 'G', 'J', 'I', 'T', '0', '2'};
bool cache_load(const std::string& file, std::vector<char>& code)
{
    if (file.empty()) return false;
    std::FILE* f = std::fopen(file.c_str(), "rb");
    if (!f) return false;
    bool ok = false;
    char magic[8];
    uint64_t len = 0, hash = 0;
    if (std::fread(magic, 1, 8, f) == 8 && std::memcmp(magic, kCacheMagic, 8) == 0 && std::fread(&len, 8, 1, f) == 1 &&
        std::fread(&hash, 8, 1, f) == 1 && len > 0 && len < (1ull << 31)) {
        code.resize((size_t)len);
        ok = std::fread(code.data(), 1, (size_t)len, f) == (size_t)len && std::fgetc(f) == EOF &&
             fnv1a(code.data(), code.size()) == hash;
    }
    std::fclose(f);
    if (!ok) code.clear();
    return ok;
}
void cache_store(const std::string& file, const std::vector<char>& code)
{
    if (file.empty() || code.empty()) return;
    const std::string tmp = file + ".tmp" + std::to_string((long long)getpid());
    std::FILE* f = std::fopen(tmp.c_str(), "wb");
    if (!f) return;                                       // a cache that cannot be written is not an error
    const uint64_t len = code.size(), hash = fnv1a(code.data(), code.size());
    const bool ok = std::fwrite(kCacheMagic, 1, 8, f) == 8 && std::fwrite(&len, 8, 1, f) == 1 && std::fwrite(&hash, 8, 1, f) == 1 &&
                    std::fwrite(code.data(), 1, code.size(), f) == code.size();
    if (std::fclose(f) != 0 || !ok || std::rename(tmp.c_str(), file.c_str()) != 0) (void)std::remove(tmp.c_str());
}
}  // namespace

int jit_compile(const std::string& src, const char* kernel_name, JitKernel& out, bool use_cache)
{
    out.ok = false;
    out.cache_file.clear();
    const std::string cached = cache_file(src);
    if (use_cache && cache_load(cached, out.code)) {
        out.name = kernel_name;
        out.log = "loaded from " + cached;
        out.cache_file = cached;
        out.ok = true;
        return 0;
    }
    if (!use_cache && !cached.empty()) (void)std::remove(cached.c_str());      // a cached object that did not load: replaced below
    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, src.c_str(), "sig_jit.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) {
        out.log = "hiprtcCreateProgram failed";
        return -1;
    }
    const hiprtcResult rc = hiprtcCompileProgram(prog, kNumCompileOptions, const_cast<const char**>(kCompileOptions));
    size_t logsz = 0;
    if (hiprtcGetProgramLogSize(prog, &logsz) == HIPRTC_SUCCESS && logsz > 1) {
        out.log.resize(logsz);
        (void)hiprtcGetProgramLog(prog, &out.log[0]);
    }
    if (rc != HIPRTC_SUCCESS) {
        (void)hiprtcDestroyProgram(&prog);
        return -2;
    }
    size_t sz = 0;
    if (hiprtcGetCodeSize(prog, &sz) != HIPRTC_SUCCESS || sz == 0) {
        (void)hiprtcDestroyProgram(&prog);
        return -3;
    }
    out.code.resize(sz);
    const hiprtcResult rc2 = hiprtcGetCode(prog, &out.code[0]);
    (void)hiprtcDestroyProgram(&prog);
    if (rc2 != HIPRTC_SUCCESS) return -4;
    cache_store(cached, out.code);
    out.name = kernel_name;
    out.ok = true;
    return 0;
}

bool jit_launch_shape_fits(int nw, int max_threads_per_block, int static_lds_bytes, int num_regs)
{
    if (nw < 1 || nw * 64 > max_threads_per_block) return false;
    if (static_lds_bytes > 64 * 1024) return false;
    // a SIMD holds 512 vector registers per lane; the nw wavefronts of a workgroup are spread over the four SIMDs of
    // a compute unit, so (nw + 3) / 4 of them share one
    const int per_simd = (nw + 3) / 4;
    return num_regs * per_simd <= 512;
}

hipError_t jit_load(JitKernel& k)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (k.fn) return k.dev == dev ? hipSuccess : hipErrorInvalidDevice;   // a word set (and its kernels) serves one device
    e = hipModuleLoadData(&k.mod, k.code.data());
    if (e != hipSuccess) return e;
    hipFunction_t fn = nullptr;
    e = hipModuleGetFunction(&fn, k.mod, k.name.c_str());
    if (e != hipSuccess) return e;
    int max_threads = 0, lds = 0, regs = 0;
    if ((e = hipFuncGetAttribute(&max_threads, HIP_FUNC_ATTRIBUTE_MAX_THREADS_PER_BLOCK, fn)) != hipSuccess) return e;
    if ((e = hipFuncGetAttribute(&lds, HIP_FUNC_ATTRIBUTE_SHARED_SIZE_BYTES, fn)) != hipSuccess) return e;
    if ((e = hipFuncGetAttribute(&regs, HIP_FUNC_ATTRIBUTE_NUM_REGS, fn)) != hipSuccess) return e;
    if (!jit_launch_shape_fits(k.nw, max_threads, lds, regs)) {
        k.log += "\nrefused: the code object does not fit the launch shape (" + std::to_string(k.nw * 64) + " threads; declares max " +
                 std::to_string(max_threads) + " threads, " + std::to_string(lds) + " bytes of LDS, " + std::to_string(regs) +
                 " registers)";
        (void)hipModuleUnload(k.mod);
        k.mod = nullptr;
        return hipErrorLaunchOutOfResources;
    }
    k.fn = fn;
    k.dev = dev;
    return hipSuccess;
}

WordSet::~WordSet()
{
    for (int dir = 0; dir < 2; ++dir)
        for (JitEntry* e : jit[dir]) {
            if (e->kernel) {
                jit_release(*e->kernel);
                delete e->kernel;
            }
            delete e;
        }
    for (int dir = 0; dir < 2; ++dir)
        for (int r = 0; r < 2; ++r)
            if (lanes[dir][r]) {
                jit_release(*lanes[dir][r]);
                delete lanes[dir][r];
            }
}

void jit_release(JitKernel& k)
{
    if (k.mod) (void)hipModuleUnload(k.mod);
    k.mod = nullptr;
    k.fn = nullptr;
}

}  // namespace sig
