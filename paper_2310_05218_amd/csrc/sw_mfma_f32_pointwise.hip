// Pointwise (1 x 1, stride 1, no padding) convolution on the matrix cores (paper, section 1.2: the pointwise stage
// of depthwise-separable convolutions; section 3: sliding sums as small matrix products).
//
//     y[n][co][p] = sum over ci of w[co][ci] * x[n][ci][p]          p = a pixel of the H x W plane
//
// With one tap there is no window: per image the sum is a plain matrix product whose B operand (channels x pixels) is
// the input tensor as it lies in memory.  The kernel therefore stages nothing of the input.  A wavefront owns 32 * QB
// consecutive pixels (counted through all images: a plane's pixel count is a multiple of QB, so the QB pixels of a lane
// never straddle two images) and CB blocks of 32 output channels.  Lane (lj, kk) of the 32 x 2 lane grid loads, for
// channel c, the QB consecutive pixels QB * lj .. QB * lj + QB - 1 with ONE load of 4 * QB bytes; element q of that
// load is its B operand for pixel block q, where block q is the pixels {QB * n + q}.  The matrix instruction does not
// care which pixel a column stands for, and on the way out the same permutation makes a lane's QB results for an
// output channel contiguous again: one 4 * QB byte store.
//
// The K index is permuted likewise: a group of eight channels is channel 4 kk + j for step j = 0..3, so the A operands
// of a lane for the four steps are four consecutive floats of a filter row, one 16-byte LDS read.  The filters of the
// workgroup's CB * 32 output channels (all of C_in) are copied to LDS once, before the first tile; after that the four
// wavefronts of a workgroup never synchronise again.  Per group of eight channels a wavefront issues 4 global loads
// and CB LDS reads for 4 * CB * QB matrix instructions (2048 cycles at CB * QB = 8); the loads run two groups ahead in
// a ring of three register sets, across tile boundaries: the next tile's first groups are requested while the current
// tile's last products run and its results are stored.
//
// Measured on 32 x 256 x 56 x 56 -> 64 (784 tiles of 128 pixels, one per wavefront): filters in LDS 3.5 us after the
// start, 33.8 us in the loop (65536 cycles of matrix instructions at the 1.94 GHz the chip holds under them: the loop
// runs at the rate of the matrix pipe), 3.8 us of stores; 46 us per launch, where the window kernels take 71.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr size_t kPwLdsMax = 150 * 1024;
constexpr int kRing = 3;      // register sets of B operands (measured: 4 and 6 are no faster)

struct PwParams {
    int C_in, C_out, HW;
    int total_px;     // N * H * W
    int tiles;        // of 32 * QB pixels
    int wpitch;       // floats between filter rows in LDS
    FastDiv by_c4;    // 16-byte groups per filter row
    Epilogue ep;
};

template <int CB, int QB, int NB>
__global__ __launch_bounds__(256, 2) void mfma_f32_pointwise_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                                    float* __restrict__ y, const PwParams P)
{
    typedef float bvec __attribute__((ext_vector_type(QB)));
    extern __shared__ __attribute__((aligned(16))) float wl[];     // [CB * 32][wpitch]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lj = lane & 31, kk = lane >> 5;
    const int co0 = blockIdx.y * (CB * 32);
    const int HW = P.HW;

    const int T = P.C_in >> 3;                               // groups of eight channels
    const int nwaves = (int)gridDim.x * 4;
    int tile = (int)blockIdx.x * 4 + wave;

    // the lane's QB pixels of a tile (a lane beyond the last pixel computes on pixel 0 and stores nothing)
    struct Place {
        bool live;
        int n, pix;
    };
    auto place = [&](int tl) __attribute__((always_inline)) {
        const int pg = tl * (32 * QB) + QB * lj;
        Place p;
        p.live = tl < P.tiles && pg < P.total_px;
        const int pgc = p.live ? pg : 0;
        p.n = pgc / HW;
        p.pix = pgc - p.n * HW;
        return p;
    };
    auto x_of = [&](const Place& p) __attribute__((always_inline)) {
        return x + ((int64_t)p.n * P.C_in + 4 * kk) * HW + p.pix;      // channel 4 kk of group 0
    };

    bvec b[NB][4];
    // group g of the tile whose lane pointer is src0, into register set `buf`
    auto fetch = [&](int buf, const float* src0, int g) __attribute__((always_inline)) {
        const int gc = g < T ? g : T - 1;
        const float* src = src0 + (int64_t)(8 * gc) * HW;
#pragma unroll
        for (int j = 0; j < 4; ++j) b[buf][j] = *reinterpret_cast<const bvec*>(src + j * HW);
    };

    // the first tile's first three groups are on their way while the filters are copied
    Place cur = place(tile);
    const float* xp = x_of(cur);
#pragma unroll
    for (int i = 0; i < NB; ++i) fetch(i, xp, i);

    // filters: rows co0 .. co0 + CB * 32 - 1 (zero beyond C_out), 16 bytes at a time, eight loads in flight per thread
    {
        const int c4 = P.C_in >> 2, total = CB * 32 * c4;
#pragma unroll 1
        for (int i0 = tid; i0 < total; i0 += 8 * 256) {
            floatx4 v[8];
            int at[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + 256 * u, ic = i < total ? i : total - 1;
                const int row = fast_div(ic, P.by_c4), g = ic - row * c4;
                at[u] = i < total ? row * P.wpitch + 4 * g : -1;
                const int rc = co0 + row < P.C_out ? co0 + row : P.C_out - 1;
                v[u] = *reinterpret_cast<const floatx4*>(w + (int64_t)rc * P.C_in + 4 * g);
                if (co0 + row >= P.C_out) v[u] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (at[u] >= 0) *reinterpret_cast<floatx4*>(wl + at[u]) = v[u];
        }
    }
    __syncthreads();

    const float* arow = wl + lj * P.wpitch + 4 * kk;         // + cb * 32 * wpitch + 8 t
    const int T3 = T - T % NB;          // groups taken by whole trips of the main loop
#pragma unroll 1
    for (; tile < P.tiles; tile += nwaves) {
        // the wavefront's next tile: its first groups are requested while this one's last products run and its
        // results leave, so the register sets are full again when the next turn starts
        const Place nxt = place(tile + nwaves);
        const float* xq = x_of(nxt);

        floatx16 acc[CB][QB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q = 0; q < QB; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[cb][q][v] = 0.f;

        auto read_a = [&](floatx4 (&a)[CB], int t) __attribute__((always_inline)) {
            const int tc = t < T ? t : T - 1;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) a[cb] = *reinterpret_cast<const floatx4*>(arow + cb * 32 * P.wpitch + 8 * tc);
        };
        auto multiply = [&](const floatx4 (&a)[CB], int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < QB; ++q)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[cb][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cb][j], b[buf][j][q], acc[cb][q], 0, 0, 0);
        };
        // group t of this tile, or, past its last group, group `buf` of the next tile (when the group count is a
        // multiple of NB that is exactly what set `buf` has to hold next; otherwise the groups left over after the
        // loop still need the first sets, and the next tile is requested behind them)
        auto fetch_on = [&](int buf, int t) __attribute__((always_inline)) {
            if (T3 == T && t >= T) fetch(buf, xq, buf);
            else fetch(buf, xp, t);
        };

        floatx4 a[2][CB];
        read_a(a[0], 0);
        // NB groups per trip, so that the register sets keep their names
#pragma unroll 1
        for (int t = 0; t < T3; t += NB) {
            // (the fences keep each group's loads where they are written: right behind the products that freed their
            // registers, NB - 1 groups ahead of their use)
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                read_a(a[(i + 1) & 1], t + i + 1);
                multiply(a[i & 1], i);
                __builtin_amdgcn_sched_barrier(0);
                fetch_on(i, t + NB + i);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (NB & 1) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) a[0][cb] = a[1][cb];
            }
        }
        if (T3 < T) {
#pragma unroll
            for (int i = 0; i < NB - 1; ++i) {
                if (T3 + i < T) {
                    read_a(a[(i + 1) & 1], T3 + i + 1);
                    multiply(a[i & 1], i);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NB; ++i) fetch(i, xq, i);
            __builtin_amdgcn_sched_barrier(0);
        }

        // register v of a lane is output channel 8 (v / 4) + 4 kk + v % 4 of the block, pixels QB lj .. QB lj + QB - 1
        if (cur.live) {
            // (the store addresses are computed here, per tile, not kept in registers the products need: the empty
            // statement hides from the compiler that they are the same for every tile)
            int pix_out = cur.pix, kk_out = kk;
            asm volatile("" : "+v"(pix_out), "+v"(kk_out));
            float* yp = y + (int64_t)cur.n * P.C_out * HW + pix_out;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int co = co0 + cb * 32 + 8 * (v >> 2) + 4 * kk_out + (v & 3);
                    if (co < P.C_out) {
                        bvec o;
#pragma unroll
                        for (int q = 0; q < QB; ++q) o[q] = apply_epilogue(acc[cb][q][v], co, P.ep);
                        *reinterpret_cast<bvec*>(yp + (int64_t)co * HW) = o;
                    }
                }
        }
        cur = nxt;
        xp = xq;
    }
}

struct PwPlan {
    bool ok = false;
    int CB = 0, QB = 0;
    size_t lds = 0;
};

PwPlan plan_pointwise(const Conv2dShape& s, const float* x, const float* w, const float* y)
{
    PwPlan a;
    const int64_t HW = (int64_t)s.H * s.W;
    if (s.R != 1 || s.S != 1 || s.stride != 1 || s.pad != 0 || s.C_in < 8 || s.C_in % 8 != 0) return a;
    if (HW * s.N >= (1LL << 31) - (1 << 20) || HW * s.C_in >= (1LL << 31) || reinterpret_cast<uintptr_t>(w) % 16 != 0) return a;
    const auto fits = [&](int cb) { return (size_t)cb * 32 * (s.C_in + 4) * sizeof(float) <= kPwLdsMax; };
    const auto aligned = [&](int qb) {
        return HW % qb == 0 && reinterpret_cast<uintptr_t>(x) % (4 * qb) == 0 && reinterpret_cast<uintptr_t>(y) % (4 * qb) == 0;
    };
    const auto units = [&](int cb, int qb) {
        return ((HW * s.N + 32 * qb - 1) / (32 * qb)) * ((s.C_out + 32 * cb - 1) / (32 * cb));
    };
    // (output-channel blocks, pixel blocks) of a wavefront, in order of preference (measured: 16-byte loads and stores
    // before 8-byte ones, two channel blocks per wavefront before one); the first one that leaves every SIMD of the
    // chip a tile to work on, else the smallest that applies
    static const int kVariants[][2] = {{2, 4}, {1, 4}, {2, 2}, {1, 2}};
    for (const auto& v : kVariants) {
        if (!fits(v[0]) || !aligned(v[1])) continue;
        a.CB = v[0];
        a.QB = v[1];
        a.ok = true;
        if (units(v[0], v[1]) >= 700) break;
    }
    if (a.ok) a.lds = (size_t)a.CB * 32 * (s.C_in + 4) * sizeof(float);
    return a;
}

template <int CB, int QB, int NB>
hipError_t launch_pw(const float* x, const float* w, float* y, const Conv2dShape& s, const PwPlan& a, hipStream_t st,
                     const Epilogue& ep)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_pointwise_kernel<CB, QB, NB>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPwLdsMax);
    if (attr != hipSuccess) return attr;
    PwParams P;
    P.C_in = s.C_in;
    P.C_out = s.C_out;
    P.HW = s.H * s.W;
    P.total_px = s.N * P.HW;
    P.tiles = (P.total_px + 32 * QB - 1) / (32 * QB);
    P.wpitch = s.C_in + 4;
    P.by_c4 = make_fastdiv(s.C_in / 4);
    P.ep = ep;
    const int gy = (s.C_out + CB * 32 - 1) / (CB * 32);
    // persistent: at most two workgroups per CU (one when the filters take more than half of its LDS)
    const int per_cu = a.lds <= 78 * 1024 ? 2 : 1;
    int gx = (P.tiles + 3) / 4;
    const int cap = (256 * per_cu + gy - 1) / gy;
    if (gx > cap) gx = cap;
    SW_NOTED_LAUNCH(note_kernel("mfma_f32_pointwise_kernel", CB, QB), (mfma_f32_pointwise_kernel<CB, QB, NB>), dim3((unsigned)gx, (unsigned)gy),
                    dim3(256), a.lds, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_pointwise_supported(const Conv2dShape& s, const float* x, const float* w, const float* y)
{
    return plan_pointwise(s, x, w, y).ok;
}

hipError_t launch_mfma_f32_pointwise(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                                     const Epilogue& ep)
{
    const PwPlan a = plan_pointwise(s, x, w, y);
    if (!a.ok) return hipErrorInvalidValue;
#define SW_PW(CBC, QBC) \
    if (a.CB == CBC && a.QB == QBC) return launch_pw<CBC, QBC, kRing>(x, w, y, s, a, st, ep)
    SW_PW(2, 4); SW_PW(1, 4); SW_PW(2, 2); SW_PW(1, 2);
#undef SW_PW
    return hipErrorInvalidValue;
}

}  // namespace swconv
