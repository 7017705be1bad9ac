// Kernels generated at run time (paper, section 2: a custom kernel for every filter size, generated when the
// size is known).  The precompiled library holds unrolled kernels for 3x3, 5x5 and 7x7 and run-time-extent kernels
// for everything else; here the source of a one-filter-per-plane kernel is specialised on the whole problem
// geometry (filter extent, plane size, padding, and a split of the taps into register-sized passes chosen for that
// extent), compiled with the run-time compiler, and kept in a per-process cache keyed by the geometry.
#include "swconv_internal.h"

#include "swconv.h"

#include <hip/hiprtc.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

namespace swconv {

namespace {

// the kernel's source text (csrc/jit/sliding_plane_jit.hip), embedded by the build
const char kJitSource[] =
#include "sw_jit_source.inc"
    ;

constexpr int kTile = 56;

struct JitPlan {
    int H, W, R, S, pad, stride, dil;
    int Ho, Wo;
    int kB;           // outputs per lane and axis (8 x 8 lanes cover the output plane)
    int P;            // LDS pitch in floats
    int RB, NT;       // filter rows / tap columns per pass
    int waves_per_cu; // 8 or 4
    size_t lds_bytes; // dynamic LDS request (padded so that no more than waves_per_cu workgroups fit a CU)
};

struct JitKernel {
    hipModule_t module;
    hipFunction_t fn;
    JitPlan plan;
    int cus;          // compute units of the device the module was loaded on
};

typedef std::tuple<int, int, int, int, int, int, int, int, int, int> JitKey;   // device, H, W, R, S, pad, stride, dil, RB, NT

std::mutex g_mutex;
std::map<JitKey, JitKernel> g_cache;
std::string g_log;

// Geometry the generated kernel covers; fills the plan.  Everything else runs the precompiled kernels.
bool jit_plan(int H, int W, int R, int S, int stride, int pad, int dil, JitPlan* out)
{
    if (stride < 1 || stride > 2 || dil < 1 || R < 1 || S < 1 || R > 64 || S > 64 || pad < 0) return false;
    const int64_t span_r = (int64_t)(R - 1) * dil + 1, span_s = (int64_t)(S - 1) * dil + 1;
    if (span_r > 64 || span_s > 64) return false;
    const int Ho = (H + 2 * pad - (int)span_r) / stride + 1, Wo = (W + 2 * pad - (int)span_s) / stride + 1;
    if (H + 2 * pad < span_r || W + 2 * pad < span_s) return false;
    if (Ho < 1 || Wo < 1 || Ho > kTile || Wo > kTile || Ho > H || Wo > W) return false;
    if (W % 4 != 0 || Wo % 4 != 0) return false;
    if ((int64_t)H * W > 4096) return false;                 // 16 16-byte groups per lane in flight at most
    JitPlan p;
    p.H = H; p.W = W; p.R = R; p.S = S; p.pad = pad; p.stride = stride; p.dil = dil; p.Ho = Ho; p.Wo = Wo;
    // the 8 x 8 lanes own kB x kB outputs each: the smallest kB that covers the output plane
    const int big = Ho > Wo ? Ho : Wo;
    p.kB = (big + 7) / 8;
    if (p.kB < 2) return false;                              // (planes below 9 x 9: the small-plane kernels)
    const int tile = 8 * p.kB;
    if (2 * Ho * Wo < tile * tile) return false;             // most lanes of the 8 x 8 grid would idle
    const int pad_up = (pad + 3) & ~3, shift = pad_up - pad;
    int need = shift + (tile - 1) * stride + (int)span_s;
    if (pad_up + W > need) need = pad_up + W;
    // kB * stride * pitch = 8 or 24 (mod 32) keeps the 8 x 4 lanes served together on 32 distinct LDS banks when
    // kB * stride is odd; other geometries take the same residue
    int P = (need + 3) & ~3;
    while (P % 16 != 8) P += 4;
    p.P = P;
    int rows = (tile - 1) * stride + (int)span_r;
    if (pad + H > rows) rows = pad + H;
    const size_t bytes = (size_t)rows * P * sizeof(float);
    if (bytes <= 20 * 1024) {
        p.waves_per_cu = 8;
        p.lds_bytes = bytes < 18432 ? 18432 : bytes;         // more than 160 KB / 9
    } else if (bytes <= 37 * 1024) {                         // beyond, the run-time-extent kernel is as fast
        p.waves_per_cu = 4;
        p.lds_bytes = bytes < 33792 ? 33792 : bytes;         // more than 160 KB / 5
    } else {
        return false;
    }
    // taps of a pass live in scalar registers: a whole filter of up to 49 taps, else about forty of them (more
    // would spill inside the loops over passes); passes of equal size on both axes.  An input row of a pass
    // ((kB - 1) * stride + (NT - 1) * dil + 1 floats, twice: the next row is in flight) must stay in registers too.
    const int row_budget = 28 - ((p.kB - 1) * stride + 1);
    int nt_max = row_budget > 0 ? row_budget / dil + 1 : 1;
    if (nt_max > 10) nt_max = 10;
    if (nt_max < 1) nt_max = 1;
    const int s_chunks = (S + nt_max - 1) / nt_max;
    p.NT = (S + s_chunks - 1) / s_chunks;
    int RB = R * S <= 49 && p.NT == S ? R : 40 / p.NT;
    if (RB < 1) RB = 1;
    if (RB > R) RB = R;
    const int r_blocks = (R + RB - 1) / RB;
    p.RB = (R + r_blocks - 1) / r_blocks;
    *out = p;
    return true;
}

int compile_plan(const JitPlan& p, std::vector<char>* code)
{
    hiprtcProgram prog;
    if (hiprtcCreateProgram(&prog, kJitSource, "sliding_plane_jit.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS)
        return SW_ERR_JIT;
    std::vector<std::string> opts = {
        "--offload-arch=gfx950", "-O3", "-std=c++17",
        // packed-FP32 VALU forms are switched off, as for every precompiled kernel
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-DSW_R=" + std::to_string(p.R), "-DSW_S=" + std::to_string(p.S), "-DSW_PAD=" + std::to_string(p.pad),
        "-DSW_H=" + std::to_string(p.H), "-DSW_W=" + std::to_string(p.W), "-DSW_P=" + std::to_string(p.P),
        "-DSW_RB=" + std::to_string(p.RB), "-DSW_NT=" + std::to_string(p.NT),
        "-DSW_STRIDE=" + std::to_string(p.stride), "-DSW_DIL=" + std::to_string(p.dil), "-DSW_KB=" + std::to_string(p.kB),
        "-DSW_MIN_WAVES=" + std::to_string(p.waves_per_cu / 4),
    };
    std::vector<const char*> argv;
    for (const std::string& o : opts) argv.push_back(o.c_str());
    const hiprtcResult rc = hiprtcCompileProgram(prog, (int)argv.size(), argv.data());
    size_t log_size = 0;
    if (hiprtcGetProgramLogSize(prog, &log_size) == HIPRTC_SUCCESS && log_size > 1) {
        g_log.assign(log_size, '\0');
        hiprtcGetProgramLog(prog, &g_log[0]);
        if (rc != HIPRTC_SUCCESS || getenv("SWCONV_JIT_VERBOSE")) fprintf(stderr, "swconv jit: %s\n", g_log.c_str());
    }
    if (rc != HIPRTC_SUCCESS) {
        hiprtcDestroyProgram(&prog);
        return SW_ERR_JIT;
    }
    size_t size = 0;
    if (hiprtcGetCodeSize(prog, &size) != HIPRTC_SUCCESS || size == 0) {
        hiprtcDestroyProgram(&prog);
        return SW_ERR_JIT;
    }
    code->resize(size);
    const hiprtcResult got = hiprtcGetCode(prog, code->data());
    hiprtcDestroyProgram(&prog);
    return got == HIPRTC_SUCCESS ? SW_OK : SW_ERR_JIT;
}

// Looks the geometry up, compiling and loading it on a miss.  SW_ERR_JIT: the compiler refused the source;
// SW_ERR_LAUNCH: no device, or the module did not load.
int get_kernel(const JitPlan& p, JitKernel* out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SW_ERR_LAUNCH;
    }
    const JitKey key(dev, p.H, p.W, p.R, p.S, p.pad, p.stride, p.dil, p.RB, p.NT);
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) {
        *out = it->second;
        return SW_OK;
    }
    std::vector<char> code;
    const int rc = compile_plan(p, &code);
    if (rc != SW_OK) return rc;
    JitKernel k;
    k.plan = p;
    if (hipModuleLoadData(&k.module, code.data()) != hipSuccess) {
        (void)hipGetLastError();
        return SW_ERR_LAUNCH;
    }
    if (hipModuleGetFunction(&k.fn, k.module, "sliding_plane_jit") != hipSuccess) {
        (void)hipGetLastError();
        (void)hipModuleUnload(k.module);
        return SW_ERR_LAUNCH;
    }
    k.cus = 256;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) k.cus = n;
    g_cache[key] = k;
    *out = k;
    return SW_OK;
}

}  // namespace

bool jit_plane_supported(const float* x, const float* y, int H, int W, int R, int S, int stride, int pad, int dil)
{
    JitPlan p;
    return reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
           jit_plan(H, W, R, S, stride, pad, dil, &p);
}

int jit_prepare_plane(int H, int W, int R, int S, int stride, int pad, int dil)
{
    JitPlan p;
    if (!jit_plan(H, W, R, S, stride, pad, dil, &p)) return SW_ERR_UNSUPPORTED;
    JitKernel k;
    return get_kernel(p, &k);
}

// Compiles the geometry without loading it (needs no device): the check that the source builds for a shape.
int jit_compile_only(int H, int W, int R, int S, int stride, int pad, int dil)
{
    JitPlan p;
    if (!jit_plan(H, W, R, S, stride, pad, dil, &p)) return SW_ERR_UNSUPPORTED;
    std::vector<char> code;
    std::lock_guard<std::mutex> lock(g_mutex);
    return compile_plan(p, &code);
}

int jit_cached_kernels()
{
    std::lock_guard<std::mutex> lock(g_mutex);
    return (int)g_cache.size();
}

int jit_launch_plane(const float* x, const float* w, float* y, int64_t planes, int planes_per_x, int n_filters, int H,
                     int W, int R, int S, int stride, int pad, int dil, hipStream_t st)
{
    JitPlan p;
    if (!jit_plan(H, W, R, S, stride, pad, dil, &p) || planes > 2147483647LL) return SW_ERR_UNSUPPORTED;
    JitKernel k;
    const int rc = get_kernel(p, &k);
    if (rc != SW_OK) return rc;
    const int64_t want = (int64_t)k.cus * k.plan.waves_per_cu;
    unsigned grid = (unsigned)(planes < want ? planes : want);
    int planes_i = (int)planes, wgs = (int)grid;
    void* args[] = {(void*)&x, (void*)&w,           (void*)&y,        (void*)&planes_i,
                    (void*)&planes_per_x, (void*)&n_filters, (void*)&wgs};
    note_kernel("sliding_plane_jit_kernel", R, S, stride, dil);
    const hipError_t e = hipModuleLaunchKernel(k.fn, grid, 1, 1, 64, 1, 1, (unsigned)k.plan.lds_bytes, st, args, nullptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return SW_ERR_LAUNCH;
    }
    return SW_OK;
}

}  // namespace swconv
