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

#include <cstdio>
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
    o << "#define EPW ((T * D + NW - 1) / NW)\n";
    o << "#define LP 65\n";
    o << R"SRC(
// increments of one tile for the 64 paths of the workgroup: tile[(tt * D + i) * 64 + lane]; every wavefront
// fetches a share of the (segment, letter) pairs one tile ahead into registers and parks them in LDS later
// (not inlined: the same code in every unit function would dominate the compile time)
__device__ __attribute__((noinline)) void tile_fetch(const float* __restrict__ X, long L, long j0, int wib, float (&r)[EPW])
{
#pragma unroll
    for (int q = 0; q < EPW; ++q) {
        int e = wib + q * NW;
        if (e >= T * D) e = T * D - 1;
        const long jj = j0 + e / D;
        const long jc = jj < 0 ? 0 : (jj < L ? jj : L - 1);
        const int i = e % D;
        const float x1 = X[(jc + 1) * D + i], x0 = X[jc * D + i];
        r[q] = (jj >= 0 && jj < L) ? x1 - x0 : 0.0f;
    }
}
__device__ __attribute__((noinline)) void tile_stage(float* tile, int lane, int wib, const float (&r)[EPW])
{
#pragma unroll
    for (int q = 0; q < EPW; ++q) {
        const int e = wib + q * NW;
        if (e < T * D) tile[e * 64 + lane] = r[q];
    }
}
)SRC";
    if (!backward) {
        o << R"SRC(
// a wavefront without a unit still takes part in loading the tiles and in the barriers
__device__ __attribute__((noinline)) void idle_unit(const float* __restrict__ X, long L, float* tile, int lane, int wib)
{
    float r[EPW];
    tile_fetch(X, L, 0, wib, r);
    tile_stage(tile, lane, wib, r);
    __syncthreads();
    for (long j0 = 0; j0 < L; j0 += T) {
        tile_fetch(X, L, j0 + T, wib, r);
        __syncthreads();
        tile_stage(tile, lane, wib, r);
        __syncthreads();
    }
}
)SRC";
    } else {
        o << R"SRC(
// gradient tile gt[(tt * D + i) * LP + lane], shared by the units of the workgroup; flushed per tile with one
// path per pass so that (segment, letter) runs are contiguous in gdx
__device__ __attribute__((noinline)) void grad_flush(float* gt, float* gdx, long L, long j0, long b0, long B, int lane, int wib)
{
    for (int bb = wib; bb < 64; bb += NW) {
        if (b0 + bb < B) {
            float* dst = gdx + ((b0 + bb) * L + j0) * D;
            for (int e = lane; e < T * D; e += 64)
                if (j0 + e / D < L) unsafeAtomicAdd(dst + e, gt[e * LP + bb]);
        }
    }
}
__device__ __attribute__((noinline)) void grad_zero(float* gt, int tid)
{
    for (int e = tid; e < T * D * LP; e += NW * 64) gt[e] = 0.0f;
}
__device__ __attribute__((noinline)) void idle_unit(const float* __restrict__ X, long L, float* tile, float* gt, float* gdx,
                                                    long b0, long B, int lane, int wib)
{
    float r[EPW];
    const long ntiles = (L + T - 1) / T;
    grad_zero(gt, wib * 64 + lane);
    tile_fetch(X, L, (ntiles - 1) * T, wib, r);
    for (long n = ntiles - 1; n >= 0; --n) {
        __syncthreads();
        tile_stage(tile, lane, wib, r);
        __syncthreads();
        tile_fetch(X, L, (n - 1) * T, wib, r);
        __syncthreads();
        grad_flush(gt, gdx, L, n * T, b0, B, lane, wib);
        __syncthreads();
        grad_zero(gt, wib * 64 + lane);
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
    o << "__device__ __attribute__((noinline)) void fwd_unit_" << uidx
      << "(const float* __restrict__ X, long L, float* tile, int lane, int wib, float* __restrict__ out)\n{\n";
    o << "    float";
    for (int r = 0; r < ud.n_slots; ++r) o << (r ? ", " : " ") << "s" << r << " = 0.0f";
    o << ";\n";
    o << "    float r[EPW];\n    tile_fetch(X, L, 0, wib, r);\n    tile_stage(tile, lane, wib, r);\n    __syncthreads();\n";
    o << "    for (long j0 = 0; j0 < L; j0 += T) {\n";
    o << "        tile_fetch(X, L, j0 + T, wib, r);\n";
    o << "        const int nt = (L - j0) < T ? (int)(L - j0) : T;\n";
    o << "        for (int tt = 0; tt < nt; ++tt) {\n";
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
    o << "        }\n        __syncthreads();\n        tile_stage(tile, lane, wib, r);\n        __syncthreads();\n    }\n";
    o << "    if (out) {\n";
    for (int r = 0; r < ud.n_slots; ++r) {
        const int32_t w = plan.slot_word[(size_t)(ud.slot_off + r)];
        if (w >= 0) o << "        out[" << w << "] = s" << r << ";\n";
    }
    o << "    }\n}\n\n";
}

void emit_backward_unit(std::ostringstream& o, const Plan& plan, int uidx)
{
    const UnitDesc& ud = plan.units[(size_t)uidx];
    const Uses uses = collect_uses(plan, ud);
    o << "__device__ __attribute__((noinline)) void bwd_unit_" << uidx
      << "(const float* __restrict__ X, long L, float* tile, float* gt, float* gdx, long b0, long B, int lane, int wib,\n"
         "     const float* __restrict__ cf, const float* __restrict__ gr)\n{\n";
    for (int r = 0; r < ud.n_slots; ++r) {
        const int32_t w = plan.slot_word[(size_t)(ud.slot_off + r)];
        const int32_t wi = w >= 0 ? w : ~w;
        o << "    float s" << r << " = cf[" << wi << "], ab" << r << " = ";
        if (w >= 0) o << "gr[" << wi << "];\n";
        else o << "0.0f;\n";
    }
    o << "    float r[EPW];\n    const long ntiles = (L + T - 1) / T;\n    grad_zero(gt, wib * 64 + lane);\n";
    o << "    tile_fetch(X, L, (ntiles - 1) * T, wib, r);\n";
    o << "    for (long n = ntiles - 1; n >= 0; --n) {\n";
    o << "        __syncthreads();\n        tile_stage(tile, lane, wib, r);\n        __syncthreads();\n";
    o << "        tile_fetch(X, L, (n - 1) * T, wib, r);\n";
    o << "        for (int tt = T - 1; tt >= 0; --tt) {\n";
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
            if (k == 1) {
                o << "            " << s << " -= dx" << i << ";\n";
                o << "            g" << i << " += " << b << ";\n";
            } else {
                o << "            " << s << " = __builtin_fmaf(-dx" << i << ", m" << k - 1 << "_1, " << s << ");\n";
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
    o << "            float* gp = gt + tt * D * LP + lane;\n";
    for (int i : uses.letters)
        o << "            __hip_atomic_fetch_add(gp + " << i << " * LP, g" << i << ", __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);\n";
    o << "        }\n";
    o << "        __syncthreads();\n        grad_flush(gt, gdx, L, n * T, b0, B, lane, wib);\n        __syncthreads();\n";
    o << "        grad_zero(gt, wib * 64 + lane);\n    }\n}\n\n";
}

}  // namespace

std::string jit_forward_source(const WordSet& ws, const Plan& plan, int NW, int T)
{
    std::ostringstream o;
    emit_prelude(o, ws.d, T, NW, false);
    const int nu = (int)plan.units.size();
    for (int u = 0; u < nu; ++u) emit_forward_unit(o, plan, u);
    o << "extern \"C\" __global__ __launch_bounds__(NW * 64) void sig_fwd_jit(const float* __restrict__ path, long B, long P,\n"
         "                                                                  float* __restrict__ coeffs, long nW)\n{\n";
    o << "    __shared__ float tile[T * D * 64];\n";
    o << "    const int lane = threadIdx.x & 63;\n    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
    o << "    const long b = (long)blockIdx.y * 64 + lane;\n    const bool valid = b < B;\n";
    o << "    const float* X = path + (valid ? b : B - 1) * P * D;\n    const long L = P - 1;\n";
    o << "    float* out = valid ? coeffs + b * nW : nullptr;\n";
    o << "    const int unit = blockIdx.x * NW + wib;\n    switch (unit) {\n";
    for (int u = 0; u < nu; ++u) o << "        case " << u << ": fwd_unit_" << u << "(X, L, tile, lane, wib, out); break;\n";
    o << "        default: idle_unit(X, L, tile, lane, wib); break;\n    }\n}\n";
    return o.str();
}

std::string jit_backward_source(const WordSet& ws, const Plan& plan, int NW, int T)
{
    std::ostringstream o;
    emit_prelude(o, ws.d, T, NW, true);
    const int nu = (int)plan.units.size();
    for (int u = 0; u < nu; ++u) emit_backward_unit(o, plan, u);
    o << "extern \"C\" __global__ __launch_bounds__(NW * 64) void sig_bwd_jit(const float* __restrict__ path,\n"
         "        const float* __restrict__ coeffs, const float* __restrict__ grad, long B, long P, long nW, float* gdx)\n{\n";
    o << "    __shared__ float tile[T * D * 64];\n    __shared__ float gt[T * D * LP];\n";
    o << "    const int lane = threadIdx.x & 63;\n    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
    o << "    const long b0 = (long)blockIdx.y * 64;\n    const long b = b0 + lane;\n    const long bc = b < B ? b : B - 1;\n";
    o << "    const float* X = path + bc * P * D;\n    const long L = P - 1;\n";
    o << "    const float* cf = coeffs + bc * nW;\n    const float* gr = grad + bc * nW;\n";
    o << "    const int unit = blockIdx.x * NW + wib;\n    switch (unit) {\n";
    for (int u = 0; u < nu; ++u)
        o << "        case " << u << ": bwd_unit_" << u << "(X, L, tile, gt, gdx, b0, B, lane, wib, cf, gr); break;\n";
    o << "        default: idle_unit(X, L, tile, gt, gdx, b0, B, lane, wib); break;\n    }\n}\n";
    return o.str();
}

int jit_compile(const std::string& src, const char* kernel_name, JitKernel& out)
{
    out.ok = false;
    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, src.c_str(), "sig_jit.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) {
        out.log = "hiprtcCreateProgram failed";
        return -1;
    }
    const char* opts[] = {"--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult rc = hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts);
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
    out.name = kernel_name;
    out.ok = true;
    return 0;
}

hipError_t jit_load(JitKernel& k)
{
    if (k.fn) return hipSuccess;
    hipError_t e = hipModuleLoadData(&k.mod, k.code.data());
    if (e != hipSuccess) return e;
    return hipModuleGetFunction(&k.fn, k.mod, k.name.c_str());
}

WordSet::~WordSet()
{
    for (int dir = 0; dir < 2; ++dir)
        for (JitKernel* k : jit[dir])
            if (k) {
                jit_release(*k);
                delete k;
            }
}

void jit_release(JitKernel& k)
{
    if (k.mod) (void)hipModuleUnload(k.mod);
    k.mod = nullptr;
    k.fn = nullptr;
}

}  // namespace sig
