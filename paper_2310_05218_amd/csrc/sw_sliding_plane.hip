// 2-D sliding window sums with one filter per plane, stride 1: single-channel convolution and
// depthwise convolution (paper, section 2: 2-D sliding convolution, fixed-size "custom" kernels
// beside a generic one; section 1.2: depthwise stage of separable convolutions).
//
// One wavefront owns a 56 x 56 output tile of one plane.  It brings the tile's input window
// (tile + filter halo, zero-filled outside the image: that is the padding) from HBM into LDS once
// with coalesced 16-byte loads.  The 64 lanes form an 8 x 8 grid; each lane owns a 7 x 7 block of
// outputs held in 49 registers.  For every input row of its window the lane reads 7 + S - 1
// values from LDS once and accumulates them into every output row and tap column they belong to:
// the horizontal shift of the window is a register rename, the vertical shift is the choice of
// accumulator row.  Filter taps are wave-uniform and sit in scalar registers.  The finished tile
// goes back through LDS so that it leaves as coalesced 16-byte stores.
//
// LDS pitches are chosen so that the 8 x 4 lanes served together hit 32 distinct banks:
// lane (bx, by) reads float 7*bx + 7*pitch*by + const, and 7*pitch = 8 or 24 (mod 32) makes the four
// by-translates of {0,7,14,21,28,3,10,17} disjoint.  72 and 104 (= 8 mod 32) serve the input
// window, 56 (= 24 mod 32) the output tile.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kB = 7;            // outputs per lane per axis
constexpr int kTile = 8 * kB;    // 56 outputs per tile per axis
constexpr int kMaxRS = 17;       // largest filter extent of the first generic kernel
constexpr int kMaxRSWide = 51;   // largest filter extent of the second one (a wider LDS window)
constexpr int kOutPitch = kTile;
constexpr int kWholeSlots = (kTile * kTile / 4 + 63) / 64;     // 16-byte groups of a plane per lane, whole-plane kernel
constexpr int kWholeSlotsBf16 = (kTile * kTile / 8 + 63) / 64; // groups of eight bf16 per lane

constexpr int in_pitch(int S) { return (3 + kTile + S - 1) <= 72 ? 72 : (3 + kTile + S - 1) <= 104 ? 104 : 136; }
constexpr int in_rows(int R) { return kTile + R - 1; }


// The lane's 7 x 7 outputs for a filter extent known at compile time.  Input row ir of the lane's
// window is read once (7 + S - 1 floats) and used by every output row orow with 0 <= ir - orow < R.
// DIL: input positions between neighbouring taps; filter row r then meets input row orow + r * DIL.
template <int R, int S, int P, int DIL = 1>
__device__ __forceinline__ void accumulate_block(const float* __restrict__ win, const float* __restrict__ wf,
                                                 float (&acc)[kB][kB])
{
    float wr[R * S];
#pragma unroll
    for (int t = 0; t < R * S; ++t) wr[t] = wf[t];
    constexpr int N = kB + (S - 1) * DIL;
    float in[2][N];
#pragma unroll
    for (int c = 0; c < N; ++c) in[0][c] = win[c];
#pragma unroll
    for (int ir = 0; ir < kB + (R - 1) * DIL; ++ir) {
        // the next row is on its way from LDS while this one is accumulated
        if (ir + 1 < kB + (R - 1) * DIL) {
#pragma unroll
            for (int c = 0; c < N; ++c) in[(ir + 1) & 1][c] = win[(ir + 1) * P + c];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int orow = 0; orow < kB; ++orow) {
            if (ir < orow || (ir - orow) % DIL != 0) continue;
            const int r = (ir - orow) / DIL;
            if (r >= R) continue;
#pragma unroll
            for (int q = 0; q < S; ++q)
#pragma unroll
                for (int oc = 0; oc < kB; ++oc)
                    acc[orow][oc] = fmaf(wr[r * S + q], in[ir & 1][oc + q * DIL], acc[orow][oc]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// One step of the run-time-extent kernel: filter row r, tap columns s0 .. s0+NT-1, all seven output rows.
// Only the NT taps of this step are live (scalars); output row orow reads input row orow + r of the lane's
// window (7 + NT - 1 floats, the next row already on its way) and slides it under the taps by register rename.
// An input row is read once per filter row it meets instead of once in all, which is what keeps the taps
// of any R x S out of the register file; LDS has the bandwidth to spare (one 8-byte read per 7 to 8 FMAs).
// DIL: input positions between neighbouring taps (dilation); the window row then spans 7 + (NT - 1) * DIL floats.
template <int NT, int DIL = 1>
__device__ __forceinline__ void row_step(const float* __restrict__ src, const float* __restrict__ taps, int P,
                                         float (&acc)[kB][kB])
{
    float wr[NT];
#pragma unroll
    for (int jj = 0; jj < NT; ++jj) wr[jj] = taps[jj];
    constexpr int N = kB + (NT - 1) * DIL;
    float in[2][N];
#pragma unroll
    for (int c = 0; c < N; ++c) in[0][c] = src[c];
#pragma unroll
    for (int orow = 0; orow < kB; ++orow) {
        if (orow + 1 < kB) {
#pragma unroll
            for (int c = 0; c < N; ++c) in[(orow + 1) & 1][c] = src[(orow + 1) * P + c];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jj = 0; jj < NT; ++jj)
#pragma unroll
            for (int oc = 0; oc < kB; ++oc) acc[orow][oc] = fmaf(wr[jj], in[orow & 1][oc + jj * DIL], acc[orow][oc]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// RC, SC > 0: filter extent known at compile time, one wavefront per tile; MAXRS is then the dilation (0: none).
// RC == 0: extent (R, S) at run
// time, up to MAXRS; four wavefronts share the tile's LDS window (which is what limits how many tiles a CU
// holds), each takes every fourth filter row, and the four partial 7 x 7 blocks are summed through LDS.
template <int RC, int SC, int MAXRS>
__global__ __launch_bounds__(RC > 0 ? 64 : 256) void sliding_plane_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ w,
                                                           float* __restrict__ y, int planes_per_x,
                                                           int n_filters, int H, int W, int R_rt,
                                                           int S_rt, int pad, int Ho, int Wo,
                                                           int tiles_x, int tiles_y, int x_vec_ok,
                                                           int y_vec_ok, const Epilogue ep, int dil)
{
    constexpr int DILC = RC > 0 && MAXRS > 1 ? MAXRS : 1;          // fixed extents: the dilation
    constexpr int RMAX = RC > 0 ? (RC - 1) * DILC + 1 : MAXRS;     // rows / columns the window holds beyond the tile, plus 1
    constexpr int SMAX = RC > 0 ? (SC - 1) * DILC + 1 : MAXRS;
    constexpr int P = in_pitch(SMAX);
    constexpr int F4_PER_ROW = (3 + kTile + SMAX - 1 + 3) / 4;   // 16-byte groups loaded per row
    static_assert(F4_PER_ROW * 4 <= P, "pitch too small");
    constexpr int NW = RC > 0 ? 1 : 4;                            // wavefronts per tile
    constexpr int NT = 64 * NW;
    constexpr int LDS_FLOATS = in_rows(RMAX) * P > kTile * kOutPitch ? in_rows(RMAX) * P : kTile * kOutPitch;
    static_assert(NW == 1 || LDS_FLOATS >= 2 * 64 * kB * kB, "window too small for two partial blocks");
    __shared__ __attribute__((aligned(16))) float lds[LDS_FLOATS];

    const int R = RC > 0 ? RC : R_rt;
    const int S = RC > 0 ? SC : S_rt;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int b = blockIdx.x;
    const int tx = b % tiles_x; b /= tiles_x;
    const int ty = b % tiles_y; b /= tiles_y;
    const int plane = b;
    const int row0 = ty * kTile, col0 = tx * kTile;          // first output of the tile
    const float* xp = x + (int64_t)(plane / planes_per_x) * H * W;
    const float* wf = w + (int64_t)(plane % n_filters) * R * S;
    float* yp = y + (int64_t)plane * Ho * Wo;

    // LDS (row e, column c) holds input (row0 - pad + e, gcol0 + c); gcol0 is a multiple of 4.
    const int pad_up = (pad + 3) & ~3;
    const int shift = pad_up - pad;
    const int gcol0 = col0 - pad_up;
    const int grow0 = row0 - pad;
    const int rows_in = kTile + (R - 1) * (RC > 0 ? DILC : dil);

    // (four 16-byte groups per thread go out before the first LDS write: one memory round trip per batch of four)
    for (int base = threadIdx.x; base < rows_in * F4_PER_ROW; base += NT * 4) {
        float4 v4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + NT * u;
            const int e = idx / F4_PER_ROW;
            const int c4 = idx - e * F4_PER_ROW;
            const int gr = grow0 + e;
            const int gc = gcol0 + 4 * c4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (idx < rows_in * F4_PER_ROW && gr >= 0 && gr < H && gc + 3 >= 0 && gc < W) {
                const float* src = xp + (int64_t)gr * W + gc;
                if (x_vec_ok && gc >= 0 && gc + 3 < W) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    if (gc >= 0) v.x = src[0];
                    if (gc + 1 >= 0 && gc + 1 < W) v.y = src[1];
                    if (gc + 2 >= 0 && gc + 2 < W) v.z = src[2];
                    if (gc + 3 < W) v.w = src[3];
                }
            }
            v4[u] = v;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + NT * u;
            if (idx < rows_in * F4_PER_ROW) {
                const int e = idx / F4_PER_ROW;
                *reinterpret_cast<float4*>(lds + e * P + 4 * (idx - e * F4_PER_ROW)) = v4[u];
            }
        }
    }
    __syncthreads();

    const int bx = lane & 7, by = lane >> 3;
    float acc[kB][kB];
#pragma unroll
    for (int i = 0; i < kB; ++i)
#pragma unroll
        for (int j = 0; j < kB; ++j) acc[i][j] = 0.f;

    const float* win = lds + (kB * by) * P + shift + kB * bx;   // the lane's window origin

    if (RC > 0) {
        accumulate_block<(RC > 0 ? RC : 1), (RC > 0 ? SC : 1), P, DILC>(win, wf, acc);
    } else {
        // Run-time extents: filter rows one at a time (every NW-th row in this wavefront), tap columns in
        // groups of eight.  Dilated filters (the window then holds the filter's span, (R - 1) * dil + 1 rows and
        // as many columns more): dilation 2 in groups of four taps, any other one tap at a time.
        if (dil == 2) {
            const int full2 = S & ~3, rem2 = S & 3;
#pragma unroll 1
            for (int r = wave; r < R; r += NW) {
                const float* row = win + 2 * r * P;
                const float* taps = wf + r * S;
#pragma unroll 1
                for (int s0 = 0; s0 < full2; s0 += 4) row_step<4, 2>(row + 2 * s0, taps + s0, P, acc);
                if (rem2 == 1) row_step<1, 2>(row + 2 * full2, taps + full2, P, acc);
                else if (rem2 == 2) row_step<2, 2>(row + 2 * full2, taps + full2, P, acc);
                else if (rem2 == 3) row_step<3, 2>(row + 2 * full2, taps + full2, P, acc);
            }
        } else if (dil != 1) {
#pragma unroll 1
            for (int r = wave; r < R; r += NW) {
                const float* row = win + r * dil * P;
                const float* taps = wf + r * S;
#pragma unroll 1
                for (int s0 = 0; s0 < S; ++s0) row_step<1>(row + s0 * dil, taps + s0, P, acc);
            }
        } else {
        const int full = S & ~7, rem = S & 7;
#pragma unroll 1
        for (int r = wave; r < R; r += NW) {
            const float* row = win + r * P;
            const float* taps = wf + r * S;
#pragma unroll 1
            for (int s0 = 0; s0 < full; s0 += 8) row_step<8>(row + s0, taps + s0, P, acc);
            switch (rem) {
                case 1: row_step<1>(row + full, taps + full, P, acc); break;
                case 2: row_step<2>(row + full, taps + full, P, acc); break;
                case 3: row_step<3>(row + full, taps + full, P, acc); break;
                case 4: row_step<4>(row + full, taps + full, P, acc); break;
                case 5: row_step<5>(row + full, taps + full, P, acc); break;
                case 6: row_step<6>(row + full, taps + full, P, acc); break;
                case 7: row_step<7>(row + full, taps + full, P, acc); break;
                default: break;
            }
        }
        }
    }

    __syncthreads();   // every lane has finished reading the window; reuse LDS
    if constexpr (NW == 4) {
        // partial blocks of wavefronts 2 and 3 into 0 and 1, then 1 into 0 (element k of lane l at k * 64 + l)
        float* slot = lds + (wave & 1) * (64 * kB * kB) + lane;
        if (wave >= 2) {
#pragma unroll
            for (int k = 0; k < kB * kB; ++k) slot[k * 64] = acc[k / kB][k % kB];
        }
        __syncthreads();
        if (wave < 2) {
#pragma unroll
            for (int k = 0; k < kB * kB; ++k) acc[k / kB][k % kB] += slot[k * 64];
        }
        __syncthreads();
        if (wave == 1) {
#pragma unroll
            for (int k = 0; k < kB * kB; ++k) lds[k * 64 + lane] = acc[k / kB][k % kB];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int k = 0; k < kB * kB; ++k) acc[k / kB][k % kB] += lds[k * 64 + lane];
        }
        __syncthreads();
    }
    if (wave == 0) {
        if (ep.bias != nullptr || ep.relu != 0) {      // fused-epilogue entry point: per-channel bias, rectifier
            const float eb = ep.bias ? ep.bias[plane % n_filters] : 0.f;
#pragma unroll
            for (int i = 0; i < kB; ++i)
#pragma unroll
                for (int j = 0; j < kB; ++j) {
                    const float t = acc[i][j] + eb;
                    acc[i][j] = ep.relu ? fmaxf(t, 0.f) : t;
                }
        }
#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j) lds[(kB * by + i) * kOutPitch + kB * bx + j] = acc[i][j];
    }
    __syncthreads();

    const int rows_out = min(kTile, Ho - row0);
    const int cols_out = min(kTile, Wo - col0);
    for (int idx = threadIdx.x; idx < rows_out * (kTile / 4); idx += NT) {
        const int e = idx / (kTile / 4);
        const int c = 4 * (idx - e * (kTile / 4));
        if (c >= cols_out) continue;
        const float4 v = *reinterpret_cast<const float4*>(lds + e * kOutPitch + c);
        float* dst = yp + (int64_t)(row0 + e) * Wo + col0 + c;
        if (y_vec_ok && c + 3 < cols_out) {
            *reinterpret_cast<float4*>(dst) = v;
        } else {
            dst[0] = v.x;
            if (c + 1 < cols_out) dst[1] = v.y;
            if (c + 2 < cols_out) dst[2] = v.z;
            if (c + 3 < cols_out) dst[3] = v.w;
        }
    }
}


// Whole-plane variant for planes that fit one tile (H_out, W_out <= 56, padding <= (R-1)/2, widths
// multiples of 4): the common CNN case.  A wavefront walks over several planes.  The next plane is
// fetched from HBM into registers (13 x 16 bytes per lane, one contiguous run per wavefront) while
// the current one is accumulated out of LDS; the zero halo is written once and never touched again,
// because the finished outputs are staged in the image area of the same LDS window.
// Orders the LDS traffic of a one-wavefront workgroup: LDS operations of a wavefront complete in
// order, so waiting for the LDS counter is all it takes.  Unlike __syncthreads() this does not wait
// for global loads in flight, which is what lets the next plane's fetch overlap the accumulation.
__device__ __forceinline__ void wave_lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// SQ: the plane and its output are exactly 56 x 56 (every slot count is then a compile-time constant).
// EP: a per-channel bias and a rectifier are applied while the outputs are staged (the plain variant carries no
// trace of them).
template <int R, int S, bool SQ, bool EP>
__global__ __launch_bounds__(64) void sliding_plane_full_kernel(const float* __restrict__ x,
                                                                const float* __restrict__ w,
                                                                float* __restrict__ y, int planes,
                                                                int planes_per_x, int n_filters, int H_rt,
                                                                int W_rt, int pad, int Ho_rt, int Wo_rt,
                                                                const Epilogue ep)
{
    const int H = SQ ? kTile : H_rt, W = SQ ? kTile : W_rt, Ho = SQ ? kTile : Ho_rt, Wo = SQ ? kTile : Wo_rt;
    constexpr int P = in_pitch(S);
    constexpr int ROWS = in_rows(R);
    constexpr int NSLOT = kWholeSlots;                        // 13 16-byte groups per lane at most
    __shared__ __attribute__((aligned(16))) float lds[ROWS * P];

    const int lane = threadIdx.x;
    const int pad_up = (pad + 3) & ~3;
    const int shift = pad_up - pad;
    const int W4 = W >> 2, Wo4 = Wo >> 2;
    const int n_in4 = H * W4, n_out4 = Ho * Wo4;

    // slot k of a lane is 16-byte group lane + 64*k of the plane; slots below n*_full are live in
    // every lane (a wave-uniform test), the one after that in the first n*_rem lanes.  In the 56 x 56
    // case the last slot is moved back to the plane's last 64 groups instead (it repeats 48 groups of
    // the slot before it with the same values), so that every slot is unconditional: the number of
    // loads and stores in flight is then the same on every path, and the wait for a prefetch does
    // not have to include the stores issued after it.
    const int nin_full = n_in4 >> 6, nin_rem = n_in4 & 63;
    const int nout_full = n_out4 >> 6, nout_rem = n_out4 & 63;
    auto group = [&](int k) { return SQ && k == NSLOT - 1 ? kTile * kTile / 4 - 64 + lane : lane + 64 * k; };
    auto in_live = [&](int k) { return SQ || k < nin_full || (k == nin_full && lane < nin_rem); };
    auto out_live = [&](int k) { return SQ || k < nout_full || (k == nout_full && lane < nout_rem); };
    int in_slot[NSLOT], out_slot[NSLOT];
#pragma unroll
    for (int k = 0; k < NSLOT; ++k) {
        const int f = group(k);
        const int ri = f / W4, ro = f / Wo4;
        in_slot[k] = (ri + pad) * P + pad_up + 4 * (f - ri * W4);
        out_slot[k] = (ro + pad) * P + pad_up + 4 * (f - ro * Wo4);
    }

    int plane = blockIdx.x;
    if (plane >= planes) return;

    for (int i = lane; i < ROWS * P / 4; i += 64) reinterpret_cast<float4*>(lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    const int bx = lane & 7, by = lane >> 3;
    const float* win = lds + (kB * by) * P + shift + kB * bx;
    float* stage = lds + (kB * by + pad) * P + pad_up + kB * bx;
    const bool full = SQ || ((Ho == kTile) && (Wo == kTile));

    floatx4 pre[NSLOT];
    auto fetch = [&](int pl) {
        const floatx4* src = reinterpret_cast<const floatx4*>(x + (int64_t)(pl / planes_per_x) * H * W);
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (in_live(k)) pre[k] = __builtin_nontemporal_load(src + group(k));
    };
    auto fill = [&]() {
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (in_live(k)) *reinterpret_cast<floatx4*>(lds + in_slot[k]) = pre[k];
    };

    // The loop is entered with the plane in LDS and the next one's loads in flight; a turn stores its
    // results first and only then waits for those loads, which are older than the stores.
    fetch(plane);
    fill();
    int next = plane + gridDim.x;
    if (next < planes) fetch(next);
    wave_lds_sync();
#pragma unroll 1
    for (;;) {
        // The wavefronts of a SIMD are served oldest first, which lets the older one run ahead and leaves the
        // younger one alone at the end, with nobody to fill its stalls.  A wavefront with more planes still to
        // go therefore asks for the higher issue priority: the two stay level.
        const int left = (planes - 1 - plane) / (int)gridDim.x;
        if (left >= 3) __builtin_amdgcn_s_setprio(3);
        else if (left == 2) __builtin_amdgcn_s_setprio(2);
        else if (left == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
        float acc[kB][kB];
#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j) acc[i][j] = 0.f;
        accumulate_block<R, S, P>(win, w + (int64_t)(plane % n_filters) * R * S, acc);
        wave_lds_sync();
        if (EP) {
            const float eb = ep.bias ? ep.bias[plane % n_filters] : 0.f;
#pragma unroll
            for (int i = 0; i < kB; ++i)
#pragma unroll
                for (int j = 0; j < kB; ++j) {
                    const float t = acc[i][j] + eb;
                    acc[i][j] = ep.relu ? fmaxf(t, 0.f) : t;
                }
        }

        if (full) {
#pragma unroll
            for (int i = 0; i < kB; ++i)
#pragma unroll
                for (int j = 0; j < kB; ++j) stage[i * P + j] = acc[i][j];
        } else {
#pragma unroll
            for (int i = 0; i < kB; ++i)
#pragma unroll
                for (int j = 0; j < kB; ++j)
                    if (kB * by + i < Ho && kB * bx + j < Wo) stage[i * P + j] = acc[i][j];
        }
        wave_lds_sync();
        floatx4* dst = reinterpret_cast<floatx4*>(y + (int64_t)plane * Ho * Wo);
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (out_live(k))
                __builtin_nontemporal_store(*reinterpret_cast<const floatx4*>(lds + out_slot[k]), dst + group(k));
        wave_lds_sync();

        if (next >= planes) break;
        plane = next;
        fill();
        next = plane + gridDim.x;
        if (next < planes) fetch(next);
        wave_lds_sync();
    }
}


// ---- bf16 activations, fp32 accumulation ----
// The whole-plane kernel with 16-bit planes in memory: a lane moves 16-byte groups of eight bf16 values, widens
// them to fp32 on their way into LDS (a bf16 is the upper half of an fp32: a shift) and rounds the finished fp32
// sums to bf16 (nearest, ties to even) on their way out.  Everything between is the fp32 kernel: the same window
// in LDS, the same 7 x 7 accumulation.  Half the HBM bytes per plane.
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// Two fp32 values -> two bf16 (nearest, ties to even; a in the low half): the conversion instruction of gfx950.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16_rne(float a, float b)
{
    return __builtin_bit_cast(unsigned, __builtin_convertvector(floatx2{a, b}, bf16x2));
}

// SQ: the plane and its output are exactly 56 x 56 (every slot is then unconditional, as in the fp32 kernel: the
// last slot is moved back to the plane's last 64 groups).
template <int R, int S, bool SQ>
__global__ __launch_bounds__(64) void sliding_plane_bf16_kernel(const unsigned short* __restrict__ x,
                                                                const float* __restrict__ w,
                                                                unsigned short* __restrict__ y, int planes,
                                                                int n_filters, int H_rt, int W_rt, int pad, int Ho_rt,
                                                                int Wo_rt)
{
    const int H = SQ ? kTile : H_rt, W = SQ ? kTile : W_rt, Ho = SQ ? kTile : Ho_rt, Wo = SQ ? kTile : Wo_rt;
    constexpr int P = in_pitch(S);
    constexpr int ROWS = in_rows(R);
    constexpr int NSLOT = kWholeSlotsBf16;                    // 7 groups of eight per lane at most
    __shared__ __attribute__((aligned(16))) float lds[ROWS * P];

    const int lane = threadIdx.x;
    const int pad_up = (pad + 3) & ~3;
    const int shift = pad_up - pad;
    const int W8 = W >> 3, Wo8 = Wo >> 3;
    const int n_in8 = H * W8, n_out8 = Ho * Wo8;
    const int nin_full = n_in8 >> 6, nin_rem = n_in8 & 63;
    const int nout_full = n_out8 >> 6, nout_rem = n_out8 & 63;
    auto group = [&](int k) { return SQ && k == NSLOT - 1 ? kTile * kTile / 8 - 64 + lane : lane + 64 * k; };
    auto in_live = [&](int k) { return SQ || k < nin_full || (k == nin_full && lane < nin_rem); };
    auto out_live = [&](int k) { return SQ || k < nout_full || (k == nout_full && lane < nout_rem); };
    int in_slot[NSLOT], out_slot[NSLOT];
#pragma unroll
    for (int k = 0; k < NSLOT; ++k) {
        const int f = group(k);
        const int ri = f / W8, ro = f / Wo8;
        in_slot[k] = (ri + pad) * P + pad_up + 8 * (f - ri * W8);
        out_slot[k] = (ro + pad) * P + pad_up + 8 * (f - ro * Wo8);
    }

    int plane = blockIdx.x;
    if (plane >= planes) return;

    for (int i = lane; i < ROWS * P / 4; i += 64) reinterpret_cast<float4*>(lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    const int bx = lane & 7, by = lane >> 3;
    const float* win = lds + (kB * by) * P + shift + kB * bx;
    float* stage = lds + (kB * by + pad) * P + pad_up + kB * bx;

    uintx4 pre[NSLOT];
    auto fetch = [&](int pl) __attribute__((always_inline)) {
        const uintx4* src = reinterpret_cast<const uintx4*>(x + (int64_t)pl * H * W);
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (in_live(k)) pre[k] = __builtin_nontemporal_load(src + group(k));
    };
    auto fill = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (in_live(k)) {
                floatx4 lo, hi;
                lo.x = __uint_as_float(pre[k].x << 16); lo.y = __uint_as_float(pre[k].x & 0xFFFF0000u);
                lo.z = __uint_as_float(pre[k].y << 16); lo.w = __uint_as_float(pre[k].y & 0xFFFF0000u);
                hi.x = __uint_as_float(pre[k].z << 16); hi.y = __uint_as_float(pre[k].z & 0xFFFF0000u);
                hi.z = __uint_as_float(pre[k].w << 16); hi.w = __uint_as_float(pre[k].w & 0xFFFF0000u);
                *reinterpret_cast<floatx4*>(lds + in_slot[k]) = lo;
                *reinterpret_cast<floatx4*>(lds + in_slot[k] + 4) = hi;
            }
    };

    fetch(plane);
    fill();
    int next = plane + gridDim.x;
    if (next < planes) fetch(next);
    wave_lds_sync();
#pragma unroll 1
    for (;;) {
        const int left = (planes - 1 - plane) / (int)gridDim.x;
        if (left >= 3) __builtin_amdgcn_s_setprio(3);
        else if (left == 2) __builtin_amdgcn_s_setprio(2);
        else if (left == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
        float acc[kB][kB];
#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j) acc[i][j] = 0.f;
        accumulate_block<R, S, P>(win, w + (int64_t)(plane % n_filters) * R * S, acc);
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < kB; ++i)
#pragma unroll
            for (int j = 0; j < kB; ++j)
                if (SQ || (kB * by + i < Ho && kB * bx + j < Wo)) stage[i * P + j] = acc[i][j];
        wave_lds_sync();
        uintx4* dst = reinterpret_cast<uintx4*>(y + (int64_t)plane * Ho * Wo);
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            if (out_live(k)) {
                const floatx4 lo = *reinterpret_cast<const floatx4*>(lds + out_slot[k]);
                const floatx4 hi = *reinterpret_cast<const floatx4*>(lds + out_slot[k] + 4);
                uintx4 v;
                v.x = pack_bf16_rne(lo.x, lo.y);
                v.y = pack_bf16_rne(lo.z, lo.w);
                v.z = pack_bf16_rne(hi.x, hi.y);
                v.w = pack_bf16_rne(hi.z, hi.w);
                __builtin_nontemporal_store(v, dst + group(k));
            }
        wave_lds_sync();

        if (next >= planes) break;
        plane = next;
        fill();
        next = plane + gridDim.x;
        if (next < planes) fetch(next);
        wave_lds_sync();
    }
}

}  // namespace

// dil > 1: the run-time-extent kernels, whose window must hold the filter's span (R - 1) * dil + 1
bool sliding_plane_supported(int H, int W, int R, int S, int stride, int pad, int dil)
{
    (void)H; (void)W;
    const int64_t span_r = (int64_t)(R - 1) * dil + 1, span_s = (int64_t)(S - 1) * dil + 1;
    return stride == 1 && dil >= 1 && span_r <= kMaxRSWide && span_s <= kMaxRSWide && pad >= 0;
}

// True when the persistent whole-plane kernel takes the problem (planes that fit one 56 x 56 tile).
// The input plane may be larger than its output (padding below (R-1)/2: up to 60 x 60 for 5x5 without padding); a
// lane holds at most kWholeSlots 16-byte groups of it, so the plane must fit 64 * kWholeSlots groups.
bool sliding_plane_whole(const float* x, const float* y, int H, int W, int R, int S, int pad, int Ho, int Wo)
{
    const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    const bool fixed = R == S && (R == 3 || R == 5 || R == 7);
    return fixed && aligned && Ho <= kTile && Wo <= kTile && 2 * pad <= R - 1 && W % 4 == 0 && Wo % 4 == 0 &&
           (int64_t)H * W <= 64 * 4 * kWholeSlots;
}

// Launch-latency regime: with fewer than 64 tiles (a quarter of the CUs) and a small filter the whole
// problem is a few hundred KB, nothing is bandwidth- or ALU-bound, and one wavefront walking through a
// 56 x 56 tile takes longer (8.3 us at 1x1x256x256, 3x3) than one thread per output (3.0 us).
bool sliding_plane_worthwhile(int64_t planes, int Ho, int Wo, int R, int S)
{
    const int64_t tiles = planes * ((Ho + kTile - 1) / kTile) * ((Wo + kTile - 1) / kTile);
    return tiles >= 64 || R * S > 25;
}

hipError_t launch_sliding_plane(const float* x, const float* w, float* y, int64_t planes, int planes_per_x,
                                int n_filters, int H, int W, int R, int S, int pad, int Ho, int Wo,
                                hipStream_t st, const Epilogue& ep, int dil)
{
    if (dil == 1 && sliding_plane_whole(x, y, H, W, R, S, pad, Ho, Wo) && planes <= 2147483647LL) {
        // enough wavefronts to fill the chip, each walking over several planes
        const int64_t want = 256 * 8;
        dim3 grid((unsigned)(planes < want ? planes : want)), block(64);
#define SW_FULL2(RC, SQC, EPC)                                                                               \
    SW_NOTED_LAUNCH(note_kernel("sliding_plane_full_kernel", (int)(RC), (int)(RC), (int)(SQC), (int)(EPC)), (sliding_plane_full_kernel<RC, RC, SQC, EPC>), grid, block, 0, st, x, w, y, (int)planes, \
                       planes_per_x, n_filters, H, W, pad, Ho, Wo, ep)
#define SW_FULL(RC)                                                                                          \
    do {                                                                                                     \
        if (sq && with_ep) SW_FULL2(RC, true, true);                                                         \
        else if (sq) SW_FULL2(RC, true, false);                                                              \
        else if (with_ep) SW_FULL2(RC, false, true);                                                         \
        else SW_FULL2(RC, false, false);                                                                     \
    } while (0)
        const bool sq = H == kTile && W == kTile && Ho == kTile && Wo == kTile;
        const bool with_ep = ep.bias != nullptr || ep.relu != 0;
        if (R == 3) SW_FULL(3);
        else if (R == 5) SW_FULL(5);
        else SW_FULL(7);
#undef SW_FULL
#undef SW_FULL2
        return hipGetLastError();
    }
    const int tiles_x = (Wo + kTile - 1) / kTile, tiles_y = (Ho + kTile - 1) / kTile;
    const int64_t blocks = planes * tiles_x * tiles_y;
    if (blocks > 2147483647LL) return hipErrorInvalidValue;
    const int x_vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0 && W % 4 == 0;
    const int y_vec_ok = reinterpret_cast<uintptr_t>(y) % 16 == 0 && Wo % 4 == 0;
    dim3 grid((unsigned)blocks);
#define SW_PLANE(RC, SC, MAXRS)                                                                          \
    SW_NOTED_LAUNCH(note_kernel("sliding_plane_kernel", (int)(RC), (int)(SC), (int)(MAXRS)), (sliding_plane_kernel<RC, SC, MAXRS>), grid, dim3(RC > 0 ? 64 : 256), 0, st, x, w, y, planes_per_x, \
                       n_filters, H, W, R, S, pad, Ho, Wo, tiles_x, tiles_y, x_vec_ok, y_vec_ok, ep, dil)
    const int span_r = (R - 1) * dil + 1, span_s = (S - 1) * dil + 1;
    if (dil == 1 && R == 3 && S == 3) SW_PLANE(3, 3, 0);
    else if (dil == 2 && R == 3 && S == 3) SW_PLANE(3, 3, 2);
    else if (dil == 4 && R == 3 && S == 3) SW_PLANE(3, 3, 4);
    else if (dil == 1 && R == 5 && S == 5) SW_PLANE(5, 5, 0);
    else if (dil == 1 && R == 7 && S == 7) SW_PLANE(7, 7, 0);
    else if (span_r <= kMaxRS && span_s <= kMaxRS) SW_PLANE(0, 0, kMaxRS);
    else SW_PLANE(0, 0, kMaxRSWide);
#undef SW_PLANE
    return hipGetLastError();
}

// bf16 planes: 3x3 / 5x5 / 7x7 at stride 1, planes that fit one 56 x 56 tile, rows that are whole 16-byte groups.
bool sliding_plane_bf16_supported(const void* x, const void* y, int H, int W, int R, int S, int stride, int pad, int Ho,
                                  int Wo)
{
    const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    const bool fixed = R == S && (R == 3 || R == 5 || R == 7);
    return stride == 1 && fixed && aligned && Ho <= kTile && Wo <= kTile && 2 * pad <= R - 1 && W % 8 == 0 &&
           Wo % 8 == 0 && (int64_t)H * W <= 64 * 8 * kWholeSlotsBf16;
}

hipError_t launch_sliding_plane_bf16(const unsigned short* x, const float* w, unsigned short* y, int64_t planes,
                                     int n_filters, int H, int W, int R, int pad, int Ho, int Wo, hipStream_t st)
{
    if (planes > 2147483647LL) return hipErrorInvalidValue;
    const int64_t want = 256 * 8;
    dim3 grid((unsigned)(planes < want ? planes : want)), block(64);
    const bool sq = H == kTile && W == kTile && Ho == kTile && Wo == kTile;
#define SW_BF16(RC)                                                                                               \
    do {                                                                                                          \
        if (sq)                                                                                                   \
            SW_NOTED_LAUNCH(note_kernel("sliding_plane_bf16_kernel", (int)(RC), (int)(RC), (int)(true)), (sliding_plane_bf16_kernel<RC, RC, true>), grid, block, 0, st, x, w, y, (int)planes, \
                               n_filters, H, W, pad, Ho, Wo);                                                     \
        else                                                                                                      \
            SW_NOTED_LAUNCH(note_kernel("sliding_plane_bf16_kernel", (int)(RC), (int)(RC), (int)(false)), (sliding_plane_bf16_kernel<RC, RC, false>), grid, block, 0, st, x, w, y, (int)planes, \
                               n_filters, H, W, pad, Ho, Wo);                                                     \
    } while (0)
    if (R == 3) SW_BF16(3);
    else if (R == 5) SW_BF16(5);
    else SW_BF16(7);
#undef SW_BF16
    return hipGetLastError();
}

}  // namespace swconv
