// Run-time specialised kernels (see jit.cpp).
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "wordset.hpp"

namespace sig {

struct JitKernel {
    std::vector<char> code;        // code object produced by hiprtc
    std::string name;              // kernel symbol
    std::string log;               // compiler log (warnings or errors)
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    int nw = 0;                    // wavefronts (units) per workgroup
    int tile = 0;                  // segments per LDS tile
    bool tried = false;
    bool ok = false;
};

std::string jit_forward_source(const WordSet& ws, const Plan& plan, int NW, int T);
std::string jit_backward_source(const WordSet& ws, const Plan& plan, int NW, int T);
// hiprtc: source -> gfx950 code object.  0 on success; the log is kept either way.  Needs no device.
int jit_compile(const std::string& src, const char* kernel_name, JitKernel& out);
// loads the code object into the current device context (first use)
hipError_t jit_load(JitKernel& k);
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
