// Run-time specialised kernels (see jit.cpp).
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>
#include <vector>

#include "wordset.hpp"

namespace sig {

struct JitKernel {
    std::vector<char> code;        // code object produced by hiprtc
    std::string name;              // kernel symbol
    std::string log;               // compiler log (warnings or errors)
    std::string cache_file;        // set when the code object came from the disk cache
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    int dev = -1;                  // device the module was loaded on
    int nw = 0;                    // wavefronts (units) per workgroup
    int tile = 0;                  // segments per LDS tile
    bool tried = false;
    bool ok = false;
    std::mutex m;                  // compilation and loading of this kernel; calls on other kernels do not wait for it
};

std::string jit_forward_source(const WordSet& ws, const Plan& plan, int NW, int T);
std::string jit_backward_source(const WordSet& ws, const Plan& plan, int NW, int T);
// hiprtc: source -> gfx950 code object.  0 on success; the log is kept either way.  Needs no device.
// With SIG_JIT_CACHE naming a directory the code object is looked up there first (use_cache) and stored after a
// compilation; use_cache = false removes a cached file and compiles afresh.
int jit_compile(const std::string& src, const char* kernel_name, JitKernel& out, bool use_cache = true);
// Loads the code object on the current device (first use) and checks what it declares against the launch shape:
// nw * 64 threads per workgroup, static LDS within the 64 KB a kernel may declare, the registers of nw / 4 wavefronts
// per SIMD.  A code object that does not fit is refused here (hipErrorLaunchFailure is never risked at dispatch).
hipError_t jit_load(JitKernel& k);
// the check alone, on the numbers hipFuncGetAttribute reports (host only; for tests)
bool jit_launch_shape_fits(int nw, int max_threads_per_block, int static_lds_bytes, int num_regs);
void jit_release(JitKernel& k);

// Full truncations with lanes = words (jit_lanes.cpp): a lane holds a word of length depth - R and the R levels below
// it, `lanes` = d^(depth - R) of them per path in `waves` wavefronts, nwb wavefronts per workgroup, T segments per
// gradient tile, TS segments of increments staged at a time.
struct LanesShape {
    bool ok;
    int R, T, TS, nwb;
    int64_t lanes, waves;
};
// the form for a batch of B paths; levels = 1 or 2 asks for that R (0: the cheaper one)
LanesShape lanes_shape(int d, int depth, bool backward, int64_t B, int levels);
// source of sig_fwd_lanes (backward = false) or sig_bwd_lanes for that shape
std::string lanes_source(int d, int depth, const LanesShape& s, bool backward);

}  // namespace sig
