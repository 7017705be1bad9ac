// Source text of the kernel that is compiled at run time, once per problem geometry (paper, section 2: custom
// kernels generated at run time for every filter size).  It is embedded into the library as a string and
// handed to the run-time compiler with these macros defined:
//   SW_R, SW_S      filter extent              SW_PAD        zero padding on every side
//   SW_H, SW_W      plane extent               SW_P          LDS pitch in floats
//   SW_STRIDE       output stride              SW_DIL        input positions between neighbouring taps
//   SW_KB           outputs per lane and axis (the 64 lanes form an 8 x 8 grid: 8 * SW_KB covers the output plane)
//   SW_RB, SW_NT    filter rows / tap columns accumulated per pass (the last pass of each axis takes the rest)
//   SW_MIN_WAVES    wavefronts per SIMD the register budget must allow
// One filter per plane, output at most 56 x 56, W and W_out multiples of 4.
//
// A wavefront walks over several planes.  The 64 lanes form an 8 x 8 grid, each lane owns a SW_KB x SW_KB block of
// outputs in registers (7 x 7 = 49 for a 56 x 56 plane).  The plane sits in LDS inside its zero frame; the next plane is on its way from HBM
// in registers while the current one is accumulated.  Everything the precompiled kernels decide at run time --
// filter extent, plane size, which 16-byte groups of a plane a lane moves, how the taps split into passes --
// is a constant here, so the loops over passes have fixed trip counts, the taps of a pass live in scalar
// registers, and an input row read from LDS serves every filter row of the pass.
// (uses compiler builtins only, so it needs no header)
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kB = SW_KB;
constexpr int kTile = 8 * kB;
constexpr int R = SW_R, S = SW_S, PAD = SW_PAD, H = SW_H, W = SW_W, P = SW_P, ST = SW_STRIDE, DIL = SW_DIL;
constexpr int SPAN_R = (R - 1) * DIL + 1, SPAN_S = (S - 1) * DIL + 1;       // input positions a filter spans
constexpr int Ho = (H + 2 * PAD - SPAN_R) / ST + 1, Wo = (W + 2 * PAD - SPAN_S) / ST + 1;
constexpr int ROWS_TAPS = (kTile - 1) * ST + SPAN_R;                        // rows the taps of the whole lane grid reach
constexpr int ROWS = ROWS_TAPS > PAD + H ? ROWS_TAPS : PAD + H;
constexpr int PAD_UP = (PAD + 3) & ~3, SHIFT = PAD_UP - PAD;
constexpr int W4 = W / 4, Wo4 = Wo / 4;
constexpr int N_IN4 = H * W4, N_OUT4 = Ho * Wo4;
constexpr int NSLOT_IN = (N_IN4 + 63) / 64, NSLOT_OUT = (N_OUT4 + 63) / 64;

static_assert(Ho >= 1 && Wo >= 1 && Ho <= kTile && Wo <= kTile && Ho <= H && Wo <= W, "plane out of range");
static_assert(W % 4 == 0 && Wo % 4 == 0, "rows must be whole 16-byte groups");
static_assert(SHIFT + (kTile - 1) * ST + SPAN_S <= P && PAD_UP + W <= P, "pitch too small");
static_assert(kB >= 1 && kB <= 7 && ST >= 1 && DIL >= 1, "parameters out of range");
static_assert(P % 4 == 0, "pitch must keep 16-byte groups aligned");

__device__ __attribute__((always_inline)) inline void wave_lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Filter rows r0 .. r0+RB-1 and tap columns s0 .. s0+NT-1 for the lane's block of outputs.  `src` is the lane's
// window at tap (r0, s0), `taps` the filter at (r0, s0).  Input row ir of the pass is read once and accumulated into
// every output row orow it meets (ir = orow * ST + r * DIL); the horizontal slide is a register rename.
constexpr bool row_meets(int ir, int RB)
{
    for (int orow = 0; orow < kB; ++orow) {
        const int d = ir - orow * ST;
        if (d >= 0 && d % DIL == 0 && d / DIL < RB) return true;
    }
    return false;
}

template <int RB, int NT>
__device__ __attribute__((always_inline)) inline void block_step(const float* __restrict__ src, const float* __restrict__ taps,
                                           float (&acc)[kB][kB])
{
    float wr[RB][NT];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int q = 0; q < NT; ++q) wr[r][q] = taps[r * S + q];
    constexpr int N = (kB - 1) * ST + (NT - 1) * DIL + 1;      // floats of an input row the pass touches
    constexpr int NR = (kB - 1) * ST + (RB - 1) * DIL + 1;     // input rows of the pass
    float in[2][N];
#pragma unroll
    for (int c = 0; c < N; ++c) in[0][c] = src[c];
#pragma unroll
    for (int ir = 0; ir < NR; ++ir) {
        // the next row is on its way from LDS while this one is accumulated (rows no output row meets are skipped)
        if (ir + 1 < NR && row_meets(ir + 1, RB)) {
#pragma unroll
            for (int c = 0; c < N; ++c) in[(ir + 1) & 1][c] = src[(ir + 1) * P + c];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int orow = 0; orow < kB; ++orow) {
            const int d = ir - orow * ST;
            if (d < 0 || d % DIL != 0 || d / DIL >= RB) continue;
            const int r = d / DIL;
#pragma unroll
            for (int q = 0; q < NT; ++q)
#pragma unroll
                for (int oc = 0; oc < kB; ++oc)
                    acc[orow][oc] = __builtin_fmaf(wr[r][q], in[ir & 1][oc * ST + q * DIL], acc[orow][oc]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// All tap columns of filter rows r0 .. r0+RB-1.
template <int RB>
__device__ __attribute__((always_inline)) inline void row_block(const float* __restrict__ win, const float* __restrict__ wf, int r0,
                                          float (&acc)[kB][kB])
{
    constexpr int NT = SW_NT;
    constexpr int S_MAIN = (S / NT) * NT, S_REST = S - S_MAIN;
    const float* src = win + r0 * DIL * P;
    const float* taps = wf + r0 * S;
#pragma unroll 1
    for (int s0 = 0; s0 < S_MAIN; s0 += NT) block_step<RB, NT>(src + s0 * DIL, taps + s0, acc);
    if constexpr (S_REST > 0) block_step<RB, S_REST>(src + S_MAIN * DIL, taps + S_MAIN, acc);
}

extern "C" __global__ __attribute__((amdgpu_flat_work_group_size(64, 64), amdgpu_waves_per_eu(SW_MIN_WAVES)))
void sliding_plane_jit(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y, int planes,
                       int planes_per_x, int n_filters, int wgs /* workgroups of the launch */)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];     // ROWS x P floats
    const int lane = (int)__builtin_amdgcn_workitem_id_x();

    // slot k of a lane is 16-byte group lane + 64*k of the plane; all but the last slot are live in every lane
    auto in_live = [&](int k) { return k < N_IN4 / 64 || lane < N_IN4 % 64; };
    auto out_live = [&](int k) { return k < N_OUT4 / 64 || lane < N_OUT4 % 64; };
    int in_slot[NSLOT_IN], out_slot[NSLOT_OUT];
#pragma unroll
    for (int k = 0; k < NSLOT_IN; ++k) {
        const int f = lane + 64 * k, ri = f / W4;
        in_slot[k] = (ri + PAD) * P + PAD_UP + 4 * (f - ri * W4);
    }
#pragma unroll
    for (int k = 0; k < NSLOT_OUT; ++k) {
        const int f = lane + 64 * k, ro = f / Wo4;
        out_slot[k] = (ro + PAD) * P + PAD_UP + 4 * (f - ro * Wo4);
    }

    int plane = (int)__builtin_amdgcn_workgroup_id_x();
    if (plane >= planes) return;

    // the zero frame is written once: finished outputs are staged inside the image area of the same window
    for (int i = lane; i < ROWS * P / 4; i += 64) reinterpret_cast<floatx4*>(lds)[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int bx = lane & 7, by = lane >> 3;
    const float* win = lds + (kB * by * ST) * P + SHIFT + kB * bx * ST;
    float* stage = lds + (kB * by + PAD) * P + PAD_UP + kB * bx;

    floatx4 pre[NSLOT_IN];
    auto fetch = [&](int pl) __attribute__((always_inline)) {
        const floatx4* src = reinterpret_cast<const floatx4*>(x + (long long)(pl / planes_per_x) * (H * W));
#pragma unroll
        for (int k = 0; k < NSLOT_IN; ++k)
            if (in_live(k)) pre[k] = __builtin_nontemporal_load(src + lane + 64 * k);
    };
    auto fill = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < NSLOT_IN; ++k)
            if (in_live(k)) *reinterpret_cast<floatx4*>(lds + in_slot[k]) = pre[k];
    };

    fetch(plane);
    wave_lds_sync();
    fill();
    int next = plane + wgs;
    if (next < planes) fetch(next);
    wave_lds_sync();
#pragma unroll 1
    for (;;) {
        // wavefronts of a SIMD are served oldest first; the one with more planes to go asks for the higher
        // issue priority, which keeps them level
        const int left = (planes - 1 - plane) / wgs;
        if (left >= 3) __builtin_amdgcn_s_setprio(3);
        else if (left == 2) __builtin_amdgcn_s_setprio(2);
        else if (left == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);

        float acc[kB][kB];
#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j) acc[i][j] = 0.f;
        const float* wf = w + (long long)(plane % n_filters) * (R * S);
        constexpr int RB = SW_RB;
        constexpr int R_MAIN = (R / RB) * RB, R_REST = R - R_MAIN;
#pragma unroll 1
        for (int r0 = 0; r0 < R_MAIN; r0 += RB) row_block<RB>(win, wf, r0, acc);
        if constexpr (R_REST > 0) row_block<R_REST>(win, wf, R_MAIN, acc);
        wave_lds_sync();

#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j)
                if ((Ho == kTile || kB * by + i < Ho) && (Wo == kTile || kB * bx + j < Wo)) stage[i * P + j] = acc[i][j];
        wave_lds_sync();
        floatx4* dst = reinterpret_cast<floatx4*>(y + (long long)plane * (Ho * Wo));
#pragma unroll
        for (int k = 0; k < NSLOT_OUT; ++k)
            if (out_live(k))
                __builtin_nontemporal_store(*reinterpret_cast<const floatx4*>(lds + out_slot[k]), dst + lane + 64 * k);
        wave_lds_sync();

        if (next >= planes) break;
        plane = next;
        fill();
        next = plane + wgs;
        if (next < planes) fetch(next);
        wave_lds_sync();
    }
}
