// Multi-channel convolution on channel-last tensors (fp32, bf16, IEEE half or int8) with both operands in LDS, the window brought
// in by direct-to-LDS loads (paper, section 3: every tap a small matrix product whose shift is an address; section 1.1:
// reduced precision on the same sliding sums).
//
//   x [N, H, W, C]     w [C_out, R, S, C]     y [N, H_out, W_out, C_out]     fp32 values or 16-bit patterns, fp32 sums
//
// The kernels that read their pixel operands straight from global memory (sw_mfma_bf16_nhwc.hip) or copy the window
// through registers (sw_mfma_nhwc.hip) are bound by cache-line look-ups and by the copy.  Here a load instruction takes
// whole lines: the rectangle of input pixels a tile touches (its window, padding included as out-of-range addresses that
// arrive as zeros) goes to LDS in 16-byte pieces (8 channels, fp32: 4), 64 consecutive pieces per instruction, and a lane's
// pixel operand for (pixel, tap, step) is one 16-byte LDS read at cell(pixel) + (r IW + s) dilation: the eight channels of
// its half of a v_mfma_f32_32x32x16_{bf16,f16}, or the four channels that four v_mfma_f32_32x32x2_f32 take one by one (K
// index j of lane half kq = channel 4 kq + j of the step's eight: the matrix instruction does not care which channel a K
// index stands for as long as both operands agree).  A cell's NP pieces are stored at slot = piece ^ key, key = the cell's
// 256-byte row of LDS modulo NP, which spreads the 16 cells a read serves per pass over all 64 banks whatever NP is (a
// 16-byte read is served 16 consecutive lanes at a time: measured, two lanes on one bank collide if and only if their numbers
// differ in the low four bits only).
//
// Workgroup = 32 CB output channels, persistent: it fetches the filters of its channels once ([channel][tap][C] rows as
// they lie in w, odd row pitch in pieces) and then walks over tiles of up to 128 PB output pixels (rows of one image, or
// whole small images), the window of the next (tile, chunk of channels) in flight while this one multiplies: four
// wavefronts only load, four multiply (pixel block 4b + w to wavefront w, all channel blocks).  Filters are the A operand,
// pixels the B operand: a lane of the result holds, for its pixel, groups of four consecutive output channels (fp32: one
// 16-byte store; 16-bit: 8 bytes, turned into whole 16-byte pieces through LDS where C_out allows).
//
// int8 (x, w int8; exact int32 sums): a piece is 16 channels, a step of two pieces one v_mfma_i32_32x32x32_i8.  The sums
// leave as int32 (16-byte stores, like fp32) or requantised to int8, q = clamp(rne(scale * float(sum + bias))), with the
// workgroup's biases and scales read from LDS, as 4 bytes per lane that pass through LDS into 16-byte pieces like the 16-bit
// results.
//
// Filters too large to stay in LDS whole (16-bit: 3 x 3 from 144 input channels on at 64 output channels per workgroup;
// fp32: from 72 on) travel with the window instead: every stage carries the chunk's part of the filters,
// [channel][tap][NP pieces] at an odd row pitch, fetched by the same loaders from L2 again for every tile.  The multipliers
// read them at the stage's address; all else is the same code (FS, a compile-time switch, so that the resident form pays
// nothing for it).
#include <algorithm>
#include <type_traits>

#include "swconv_internal.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

#define SW_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr size_t kLdsTotal = 156 * 1024;
constexpr size_t kFilterMax = 76 * 1024;       // resident filters of a workgroup
constexpr int kMaxWK = 12;                     // window loads per loading wavefront and stage
constexpr int kMaxFK = 12;                     // filter loads per loading wavefront and stage (filters fetched per chunk)
constexpr unsigned kBeyond = 0x80000000u;
// formats beyond Elem's: int8 operands with exact int32 sums, leaving as int32 or requantised to int8
constexpr int kFmtS8 = 3, kFmtS8Q = 4, kFormats = 5;

struct LdsParams {
    Epilogue ep;
    Requant rq;                    // (int8 -> int8)
    int rq_off;                    // (int8 -> int8) 32 CB biases, then 32 CB scales, once per workgroup
    int N, H, W, C, C_out, R, S, stride, pad, dil, Ho, Wo;
    int pix_bytes, cpt;            // bytes of a pixel's channels; 16-byte pieces of a tap in a filter row (C / 8, fp32: C / 4)
    int NI, TH, tiles_y, tiles;    // images and output rows per tile, row tiles per image, tiles in all
    int IH, IW, cells_img, WC;     // window rows and columns of one image, their product, cells of a window
    int NP, chunks;                // 16-byte pieces per pixel and chunk (2, 4 or 8), chunks of 8 NP channels
    int wloads;                    // 64-piece loads per window stage
    int frow, fpitch;              // 16-byte pieces of an output channel's filters (R S C / 8), row pitch in LDS (odd)
    int win_off, stage_bytes;      // window stages behind the filters
    int fstream;                   // the filters do not fit LDS whole: the chunk's part ([channel][tap][NP pieces], pitch fp2)
    int fp2, fs_off, fsloads;      // travels with every window stage, fs_off bytes behind the window, in fsloads loads
    int out_off;                   // per multiplying wavefront: 32 pixels x (64 CB + 16) bytes for the transposed store (< 0: none)
    unsigned x_bytes, w_bytes;
    FastDiv by_tiles_y, by_cells_img, by_IW, by_thwo, by_Wo, by_fpitch, by_fp2;
};

__device__ __forceinline__ unsigned round16_bits(float f, bool f16)
{
    if (f16) return (unsigned)__builtin_bit_cast(unsigned short, (_Float16)f);     // v_cvt_f16_f32: nearest even
    return (unsigned)__builtin_bit_cast(unsigned short, (__bf16)f);                // v_cvt_pk_bf16_f32: nearest even
}

// EK: format (Elem: fp32, bf16, IEEE half; kFmtS8, kFmtS8Q).  CB: blocks of 32 output channels per workgroup.  PB: blocks of 32 pixels per wavefront.
// KSC: steps of 16 channels per tap and chunk (NP / 2).  FS: filters per chunk with the window (else resident).
template <int EK, int CB, int PB, int KSC, bool FS>
__global__ __launch_bounds__(512, 2) void mfma_nhwc_lds_kernel(const unsigned char* __restrict__ x, const unsigned char* __restrict__ w,
                                                               unsigned char* __restrict__ yb, const LdsParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool F16 = EK == kElemF16;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int co0 = blockIdx.y * (32 * CB);
    const int steps_per_wg = ((P.tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x) * P.chunks;   // (tile, chunk) steps
    const int m = P.NP - 1, lnp = __builtin_ctz(P.NP);

    // the filters, once, by every wavefront: slot q of the filter area is piece q % fpitch of output channel q / fpitch
    if (!FS) {
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(w), 0, P.w_bytes, 0x00020000);
        const int floads = (32 * CB * P.fpitch + 63) >> 6;
#pragma unroll 1
        for (int k = wave; k < floads; k += 8) {
            const int q = 64 * k + lane;
            const int co = fast_div(q, P.by_fpitch), j = q - co * P.fpitch;
            const unsigned off = (co < 32 * CB && j < P.frow && co0 + co < P.C_out) ? (unsigned)(((co0 + co) * P.frow + j) * 16) : kBeyond;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, SW_LDS_PTR(smem + 1024 * k), 16, off, 0, 0, 0);
        }
    }
    if constexpr (EK == kFmtS8Q) {
        // the requantisation's bias and scale of the workgroup's channels (the first barrier orders them before their use)
        if (tid < 32 * CB) {
            const int co = co0 + tid;
            reinterpret_cast<int*>(smem + P.rq_off)[tid] = (P.rq.bias != nullptr && co < P.C_out) ? P.rq.bias[co] : 0;
            reinterpret_cast<float*>(smem + P.rq_off)[32 * CB + tid] = co < P.C_out ? P.rq.scale[co] : 0.f;
        }
    }
    if (wave >= 4) {
        // ---------------------------------------------------------------------------------------- the loaders
        const int lw = wave - 4;
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(x), 0, P.x_bytes, 0x00020000);
        // this lane's slot in each window load of this wavefront (loads lw, lw + 4, ...): its cell's place in the window
        // (image, row, column) and the byte offset of its piece from the tile's origin; what changes per tile is the
        // origin and which rows and images exist
        int wrow[kMaxWK], wimg[kMaxWK];
        unsigned wofs[kMaxWK];
#pragma unroll
        for (int k = 0; k < kMaxWK; ++k) {
            // (wave-uniform; the uses carry the same test.  Code that runs once costs its instruction fetches: an entry
            // is about 40 instructions, and the workgroup's first load leaves only after the last of them)
            if (lw + 4 * k >= P.wloads) continue;
            const int q = 64 * (lw + 4 * k) + lane;
            const int cell = q >> lnp, slot = q & m;                // (NP is a power of two)
            const int piece = slot ^ ((cell >> (4 - lnp)) & m);
            const int i = fast_div(cell, P.by_cells_img), rem = cell - i * P.cells_img;
            const int e = fast_div(rem, P.by_IW), f = rem - e * P.IW;
            const int gc = f - P.pad;
            const bool in = cell < P.WC && gc >= 0 && gc < P.W;
            wimg[k] = i;
            wrow[k] = in ? e : -(1 << 20);                          // (a row that never exists)
            wofs[k] = (unsigned)(((i * P.H + e) * P.W + gc) * P.pix_bytes + 16 * piece);
        }
        // (filters per chunk) this lane's slot in each filter load of this wavefront: piece j % NP of tap j / NP of output
        // channel co, j = q % fp2; byte offset in w for chunk 0
        unsigned fofs[kMaxFK];
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(w), 0, P.w_bytes, 0x00020000);
#pragma unroll
        for (int k = 0; k < kMaxFK; ++k) {
            fofs[k] = kBeyond;
            if (FS && lw + 4 * k < P.fsloads) {
                const int q = 64 * (lw + 4 * k) + lane;
                const int co = fast_div(q, P.by_fp2), j = q - co * P.fp2;
                const int tap = j >> lnp, piece = j & m;
                if (co < 32 * CB && tap < P.R * P.S && co0 + co < P.C_out)
                    fofs[k] = (unsigned)(((co0 + co) * P.R * P.S + tap) * P.pix_bytes + 16 * piece);
            }
        }
        auto issue = [&](int step, int stage) __attribute__((always_inline)) {
            const int tl = step / P.chunks, ch = step - tl * P.chunks;              // (wave-uniform)
            const int tile = (int)blockIdx.x + tl * (int)gridDim.x;
            const int ig = fast_div(tile, P.by_tiles_y), ty = tile - ig * P.tiles_y;
            const int n0 = ig * P.NI, gr0 = ty * P.TH * P.stride - P.pad;
            const unsigned origin = (unsigned)((n0 * P.H + gr0) * P.W * P.pix_bytes + ch * (16 * P.NP));
            unsigned char* sw = smem + P.win_off + stage * P.stage_bytes;
#pragma unroll
            for (int k = 0; k < kMaxWK; ++k) {
                if (lw + 4 * k < P.wloads) {
                    const int gr = gr0 + wrow[k];
                    const bool in = gr >= 0 && gr < P.H && n0 + wimg[k] < P.N;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, SW_LDS_PTR(sw + 1024 * (lw + 4 * k)), 16, in ? origin + wofs[k] : kBeyond, 0, 0, 0);
                }
            }
            if (FS) {
                const unsigned choff = (unsigned)(ch * (16 * P.NP));
#pragma unroll
                for (int k = 0; k < kMaxFK; ++k)
                    if (lw + 4 * k < P.fsloads)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, SW_LDS_PTR(sw + P.fs_off + 1024 * (lw + 4 * k)), 16,
                                                                 fofs[k] == kBeyond ? kBeyond : fofs[k] + choff, 0, 0, 0);
            }
        };
        if (steps_per_wg > 0) issue(0, 0);
#pragma unroll 1
        for (int s = 0; s < steps_per_wg; ++s) {
            __builtin_amdgcn_s_waitcnt(0);              // this wavefront's loads of step s (and the filters) have landed
            __syncthreads();                            // barrier s: step s is complete, step s - 1 has been multiplied
            if (s + 1 < steps_per_wg) issue(s + 1, (s + 1) & 1);
        }
        __builtin_amdgcn_s_waitcnt(0);
        return;
    }

    // -------------------------------------------------------------------------------------------- the multipliers
    const int lj = lane & 31, kq = lane >> 5;
    const int thwo = P.TH * P.Wo, HoWo = P.Ho * P.Wo;
    // this wavefront's pixel blocks: block 4b + wave of the tile; the pixel's cell in the window does not depend on the tile
    int cell0[PB], pl[PB];
#pragma unroll
    for (int b = 0; b < PB; ++b) {
        const int p = 32 * (4 * b + wave) + lj;
        const int pc = p < P.NI * thwo ? p : 0;
        const int i = fast_div(pc, P.by_thwo), rem = pc - i * thwo;
        const int ol = fast_div(rem, P.by_Wo), ow = rem - ol * P.Wo;
        cell0[b] = i * P.cells_img + (ol * P.IW + ow) * P.stride;
        pl[b] = p;
    }
    // A operand of (channel block cb, tap, step ks): resident filters: row pitch fpitch pieces, C / 8 pieces per tap, the
    // chunk's NP pieces at chunk NP; filters per chunk: row pitch fp2, NP pieces per tap
    const int apitch = FS ? P.fp2 : P.fpitch, cpt = FS ? P.NP : P.cpt;
    const unsigned char* arow = smem + (lj * apitch + kq) * 16;            // + 32 cb apitch 16 + (tap cpt + 2 ks) 16

    // the lane's 16 CB output channels' biases, read once (zeros without a bias); the rectifier as a lower bound
    float bias[CB][16];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int co = co0 + cb * 32 + 8 * (v >> 2) + 4 * kq + (v & 3);
            if constexpr (EK < kFmtS8) bias[cb][v] = (P.ep.bias != nullptr && co < P.C_out) ? P.ep.bias[co] : 0.f;
            else bias[cb][v] = 0.f;
        }
    const float floor_ = P.ep.relu ? 0.f : -__builtin_inff();
    auto finish32 = [&](float t, int cb, int v) __attribute__((always_inline)) { return fmaxf(t + bias[cb][v], floor_); };
    auto finish = [&](float t, int cb, int v) __attribute__((always_inline)) { return round16_bits(finish32(t, cb, v), F16); };

    using Acc = std::conditional_t<(EK >= kFmtS8), intx16, floatx16>;
    Acc acc[CB][PB];
#pragma unroll 1
    for (int s = 0; s < steps_per_wg; ++s) {
        const int tl = s / P.chunks, ch = s - tl * P.chunks;               // (wave-uniform)
        if (ch == 0) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int b = 0; b < PB; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[cb][b][v] = 0;
        }
        if (s == 0) __builtin_amdgcn_s_waitcnt(0);                         // (this wavefront's share of the filters)
        // barrier s, without the fence of __syncthreads: that would wait for the stores of the tile before to be
        // acknowledged (about 2 us per tile); nothing here reads what they wrote
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const unsigned char* sw = smem + P.win_off + (s & 1) * P.stage_bytes;
        const unsigned char* ab = FS ? arow + P.win_off + (s & 1) * P.stage_bytes + P.fs_off : arow + (ch * P.NP) * 16;
        // One tap at a time: the KSC steps of 16 channels of a tap are KSC CB PB matrix instructions on KSC (CB + PB)
        // operand reads; the reads of tap t + 1 (into the other register set) sit between the matrix instructions of
        // tap t.  Per tap the window address costs three vector instructions per block and two per read.
        const int taps = P.R * P.S;
        struct Ops {
            intx4 a[KSC][CB], b[KSC][PB];
        };
        Ops ops[2];
        int r = 0, sc = 0;
        auto read_tap = [&](Ops& o, int tap) __attribute__((always_inline)) {
            const int toff = (r * P.IW + sc) * P.dil;
            if (++sc == P.S) { sc = 0; ++r; }
            const unsigned char* at = ab + tap * cpt * 16;
#pragma unroll
            for (int ks = 0; ks < KSC; ++ks)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) o.a[ks][cb] = *reinterpret_cast<const intx4*>(at + (32 * cb * apitch + 2 * ks) * 16);
#pragma unroll
            for (int b = 0; b < PB; ++b) {
                const int cell = cell0[b] + toff;
                const unsigned char* cb_ = sw + ((cell << lnp) << 4);
                const int sw_ = (cell >> (4 - lnp)) & m;
#pragma unroll
                for (int ks = 0; ks < KSC; ++ks) o.b[ks][b] = *reinterpret_cast<const intx4*>(cb_ + (((2 * ks + kq) ^ sw_) << 4));
            }
        };
        auto multiply_tap = [&](const Ops& o) __attribute__((always_inline)) {
#pragma unroll
            for (int ks = 0; ks < KSC; ++ks) {
                if constexpr (EK == kElemF32) {
                    // a piece is four channels: matrix instruction j of the step takes channel j of the two lane halves' pieces
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int b = 0; b < PB; ++b)
#pragma unroll
                            for (int cb = 0; cb < CB; ++cb) {
                                // (the whole vector is cast, then indexed: a cast of one indexed element took element 0)
                                const floatx4 af = __builtin_bit_cast(floatx4, o.a[ks][cb]), bf = __builtin_bit_cast(floatx4, o.b[ks][b]);
                                acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc[cb][b], 0, 0, 0);
                            }
                } else if constexpr (EK >= kFmtS8) {
#pragma unroll
                    for (int b = 0; b < PB; ++b)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
                            acc[cb][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.a[ks][cb], o.b[ks][b], acc[cb][b], 0, 0, 0);
                } else {
#pragma unroll
                    for (int b = 0; b < PB; ++b)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) {
                            if constexpr (F16)
                                acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, o.a[ks][cb]),
                                                                                    __builtin_bit_cast(halfx8, o.b[ks][b]), acc[cb][b], 0, 0, 0);
                            else
                                acc[cb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o.a[ks][cb]),
                                                                                     __builtin_bit_cast(bf16x8, o.b[ks][b]), acc[cb][b], 0, 0, 0);
                        }
                }
            }
        };
        read_tap(ops[0], 0);
#pragma unroll 1
        for (int tap = 0; tap < taps; tap += 2) {
            if (tap + 1 < taps) read_tap(ops[1], tap + 1);
            __builtin_amdgcn_sched_barrier(0);
            multiply_tap(ops[0]);
            __builtin_amdgcn_sched_barrier(0);
            if (tap + 1 < taps) {
                if (tap + 2 < taps) read_tap(ops[0], tap + 2);
                __builtin_amdgcn_sched_barrier(0);
                multiply_tap(ops[1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        if (ch + 1 < P.chunks) continue;
        // ---- the tile is finished: register v of a lane is output channel 8 (v / 4) + 4 kq + v % 4 of the block
        const int tile = (int)blockIdx.x + tl * (int)gridDim.x;
        const int ig = fast_div(tile, P.by_tiles_y), ty = tile - ig * P.tiles_y;
        const int n0 = ig * P.NI, row0 = ty * P.TH;
        const int valid_px = P.NI > 1 ? min(P.NI, P.N - n0) * HoWo : min(P.TH, P.Ho - row0) * P.Wo;
        if constexpr (EK == kElemF32 || EK == kFmtS8) {
            // four consecutive output channels of a pixel are 16 bytes: stored as they lie in the accumulators
            using T = std::conditional_t<EK == kFmtS8, int, float>;
            typedef T Tx4 __attribute__((ext_vector_type(4)));
            T* y = reinterpret_cast<T*>(yb);
#pragma unroll
            for (int b = 0; b < PB; ++b) {
                if (pl[b] >= valid_px) continue;
                const int i = fast_div(pl[b], P.by_thwo), rem = pl[b] - i * thwo;       // (pixel of image n0 + i, rows from row0)
                T* yp = y + ((int64_t)(n0 + i) * HoWo + row0 * P.Wo + rem) * P.C_out;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int co = co0 + cb * 32 + 8 * q + 4 * kq;
                        if (co < P.C_out) {
                            Tx4 v;
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                if constexpr (EK == kFmtS8) v[j] = acc[cb][b][4 * q + j];
                                else v[j] = finish32(acc[cb][b][4 * q + j], cb, 4 * q + j);
                            }
                            *reinterpret_cast<Tx4*>(yp + co) = v;
                        }
                    }
            }
            continue;
        }
        // 16-bit and requantised int8 results: four consecutive output channels of a lane are 4 OB bytes
        constexpr int OB = EK == kFmtS8Q ? 1 : 2;
        using Pack = std::conditional_t<EK == kFmtS8Q, int, intx2>;
        auto pack = [&](int cb, int b, int q) __attribute__((always_inline)) {
            if constexpr (EK == kFmtS8Q) {
                // q = clamp(rne(scale * float(acc + bias)), relu ? 0 : -128, 127), every step in fp32 as the definition has it
                const int c = cb * 32 + 8 * q + 4 * kq;
                const intx4 qb = *reinterpret_cast<const intx4*>(smem + P.rq_off + 4 * c);
                const floatx4 qs = *reinterpret_cast<const floatx4*>(smem + P.rq_off + 4 * (32 * CB + c));
                const float lo_ = P.rq.relu ? 0.0f : -128.0f;
                int r = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float f = rintf(__int2float_rn((int)acc[cb][b][4 * q + j] + qb[j]) * qs[j]);
                    f = fminf(fmaxf(f, lo_), 127.0f);
                    r |= ((int)f & 255) << (8 * j);
                }
                return r;
            } else {
                unsigned h[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = finish(acc[cb][b][4 * q + j], cb, 4 * q + j);
                return intx2{(int)(h[0] | (h[1] << 16)), (int)(h[2] | (h[3] << 16))};
            }
        };
        if (P.out_off >= 0) {
            // through LDS, so that a store instruction writes whole lines: the lane's 16 CB values go to
            // [pixel][channel] rows of this wavefront's area (4 OB bytes at a time), and come back as 16-byte pieces with
            // consecutive lanes on consecutive pieces of a pixel
            constexpr int NC = 2 * CB * OB;                                 // 16-byte pieces of a pixel's channels
            constexpr int OP = 32 * CB * OB + 16;                           // row pitch
            unsigned char* lo = smem + P.out_off + wave * (32 * OP);
            const int64_t tile_px0 = (int64_t)n0 * HoWo + row0 * P.Wo;
#pragma unroll
            for (int b = 0; b < PB; ++b) {
                if (32 * (4 * b + wave) >= valid_px) continue;              // (wave-uniform)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int col = cb * 32 + 8 * q + 4 * kq;
                        *reinterpret_cast<Pack*>(lo + lj * OP + OB * col) = pack(cb, b, q);
                    }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int pass = 0; pass < NC / 2; ++pass) {
                    const int px = lane / NC + (64 / NC) * pass, piece = lane % NC;
                    const intx4 v = *reinterpret_cast<const intx4*>(lo + px * OP + 16 * piece);
                    const int p = 32 * (4 * b + wave) + px;
                    if (p < valid_px && co0 + (16 / OB) * piece < P.C_out)
                        *reinterpret_cast<intx4*>(yb + ((tile_px0 + p) * P.C_out + co0) * OB + 16 * piece) = v;
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // (the area is written again for the next block)
            }
            continue;
        }
#pragma unroll
        for (int b = 0; b < PB; ++b) {
            if (pl[b] >= valid_px) continue;
            const int i = fast_div(pl[b], P.by_thwo), rem = pl[b] - i * thwo;       // (pixel of image n0 + i, rows from row0)
            unsigned char* yp = yb + ((int64_t)(n0 + i) * HoWo + row0 * P.Wo + rem) * P.C_out * OB;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int co = co0 + cb * 32 + 8 * q + 4 * kq;
                    if (co < P.C_out) *reinterpret_cast<Pack*>(yp + co * OB) = pack(cb, b, q);
                }
        }
    }
}

struct LdsPlan {
    bool ok = false;
    int CB = 0, PB = 0;
    size_t lds = 0;
    unsigned gx = 0, gy = 0;
    double est = 0;
    int64_t tiles = 0;
    LdsParams P;
};

LdsPlan search_plan(const Conv2dShape& s, int ek, const void* x, const void* w, const void* y)
{
    LdsPlan best;
    const int RS = s.R * s.S;
    const int es = ek >= kFmtS8 ? 1 : (int)elem_size(ek), cpp = 16 / es;    // bytes of an element, channels in a 16-byte piece
    const int ob = ek == kFmtS8 ? 4 : ek == kFmtS8Q ? 1 : es;                // bytes of an output element
    const int64_t x_bytes = (int64_t)s.N * s.H * s.W * s.C_in * es, w_bytes = (int64_t)s.C_out * RS * s.C_in * es;
    // a step of the matrix instructions takes two pieces; a lane stores four consecutive output channels at once
    if (s.C_in % (2 * cpp) != 0 || s.C_out % 4 != 0 || x_bytes >= (1LL << 31) || w_bytes >= (1LL << 31)) return best;
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0 ||
        reinterpret_cast<uintptr_t>(y) % (4 * ob) != 0)
        return best;
    if ((int64_t)s.N * s.Ho * s.Wo * s.C_out >= (1LL << 40)) return best;
    const int frow = RS * s.C_in / cpp, fpitch = frow | 1;
    const int64_t IW = (int64_t)(s.Wo - 1) * s.stride + (int64_t)(s.S - 1) * s.dil + 1;
    const int HoWo = s.Ho * s.Wo;
    // the transposed store wants whole 16-byte pieces of y
    const bool wide_out = ob <= 2 && s.C_out % (16 / ob) == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    // CB blocks of 32 output channels per workgroup; filters resident (fstream = false) or fetched per chunk with the window;
    // NP pieces of eight channels per pixel and chunk: the wider the chunk, the fewer steps; the narrower, the larger the
    // tile LDS holds
    auto consider = [&](int CB, bool fstream, int PB, int NP, int NI, int tiles_y) {
        if (s.C_in % (cpp * NP) != 0) return;
        const int chunks = s.C_in / (cpp * NP);
        const int co_blocks = (s.C_out + 32 * CB - 1) / (32 * CB);
        if (co_blocks > 65535) return;
        const int fp2 = (RS * NP) | 1;
        const int64_t fsloads = fstream ? ((int64_t)32 * CB * fp2 + 63) / 64 : 0;
        if (fsloads > 4 * kMaxFK) return;
        const size_t fbytes = fstream ? 0 : ((size_t)32 * CB * fpitch * 16 + 1023) & ~(size_t)1023;
        if (fbytes > kFilterMax) return;
        const size_t obytes = (wide_out ? (size_t)4 * 32 * (32 * CB * ob + 16) : 0) + (ek == kFmtS8Q ? 512 : 0);
        const int tp_max = 128 * PB;
        const int TH = (s.Ho + tiles_y - 1) / tiles_y;
        if ((int64_t)TH * s.Wo * NI > tp_max || (s.Ho + TH - 1) / TH != tiles_y) return;
        const int64_t IH = (int64_t)(TH - 1) * s.stride + (int64_t)(s.R - 1) * s.dil + 1;
        const int64_t WC = NI * IH * IW;
        const int64_t wloads = (WC * NP + 63) / 64;
        if (wloads > 4 * kMaxWK) return;
        const size_t stage = (size_t)(wloads + fsloads) * 1024;
        const size_t lds = fbytes + 2 * stage + obytes;
        if (lds > kLdsTotal) return;
        const int64_t groups = (s.N + NI - 1) / NI;
        const int64_t tiles = groups * tiles_y;
        if (tiles > 2147483647LL) return;
        double est;
        if (es == 4) {
            // fp32: the matrix instructions bound a step (64 cycles each, four per 16-byte operand pair) unless its loads
            // take longer (about 10 bytes per clock and CU out of L2, 5 for a single tap, whose pixels come from memory
            // once); a step costs about 1500 cycles beyond them (pipeline fill, barrier), a tile its stores.  Cycles of a
            // workgroup: its tiles one after the other; more workgroups than CUs run in turns.
            const double mfma = (double)RS * (NP / 2) * 4 * CB * PB * 64;
            const double load = (double)stage / (RS == 1 ? 5.0 : 10.0);
            const double tile_cycles = chunks * (std::max(mfma + 700, load) + 800) + 900.0 * CB * PB;
            const int64_t gx = std::max<int64_t>(1, std::min<int64_t>(tiles, 256 / std::min(co_blocks, 256)));
            const double turns = std::max(1.0, (double)gx * co_blocks / 256.0);
            est = turns * (double)((tiles + gx - 1) / gx) * tile_cycles + (double)fbytes / 13.0;
        } else {
            // 16-bit: LDS operand reads bound a step.  Periods of one block through all of K: every wavefront multiplies PB
            // blocks, live or not; 256 workgroups at a time.  Two blocks per wavefront halve the filter reads per matrix
            // instruction, but with a single tap a step is too short for them to pay (measured); one channel block per
            // workgroup doubles the window reads per matrix instruction; filters per chunk are fetched again for every tile.
            est = std::max((double)PB, (double)tiles * co_blocks * PB / 256.0) * (PB == 2 ? (RS >= 4 ? 0.8 : 1.1) : 1.0) *
                  (1.0 + 0.05 * (chunks - 1)) * (CB == 1 && s.C_out > 32 ? 1.2 : 1.0) * (fstream ? 1.3 : 1.0);
        }
        if (best.ok && (est > best.est || (est == best.est && tiles >= best.tiles))) return;
        best.ok = true;
        best.CB = CB;
        best.PB = PB;
        best.lds = lds;
        best.est = est;
        best.tiles = tiles;
        best.gy = (unsigned)co_blocks;
        best.gx = (unsigned)std::max<int64_t>(1, std::min<int64_t>(tiles, 256 / std::min(co_blocks, 256)));
        LdsParams& P = best.P;
        P.N = s.N; P.H = s.H; P.W = s.W; P.C = s.C_in; P.C_out = s.C_out; P.R = s.R; P.S = s.S; P.stride = s.stride;
        P.pad = s.pad; P.dil = s.dil; P.Ho = s.Ho; P.Wo = s.Wo;
        P.pix_bytes = s.C_in * es; P.cpt = s.C_in / cpp;
        P.NI = NI; P.TH = TH; P.tiles_y = tiles_y; P.tiles = (int)tiles;
        P.IH = (int)IH; P.IW = (int)IW; P.cells_img = (int)(IH * IW); P.WC = (int)WC;
        P.NP = NP; P.chunks = chunks; P.wloads = (int)wloads;
        P.frow = frow; P.fpitch = fpitch;
        P.fstream = fstream ? 1 : 0; P.fp2 = fp2; P.fs_off = (int)(wloads * 1024); P.fsloads = (int)fsloads;
        P.win_off = (int)fbytes; P.stage_bytes = (int)stage;
        P.out_off = wide_out ? (int)(fbytes + 2 * stage) : -1;
        P.rq_off = (int)(lds - 512);
        P.x_bytes = (unsigned)x_bytes; P.w_bytes = (unsigned)w_bytes;
        P.by_tiles_y = make_fastdiv(tiles_y);
        P.by_cells_img = make_fastdiv(P.cells_img);
        P.by_IW = make_fastdiv(P.IW);
        P.by_thwo = make_fastdiv(TH * s.Wo);
        P.by_Wo = make_fastdiv(s.Wo);
        P.by_fpitch = make_fastdiv(fpitch);
        P.by_fp2 = make_fastdiv(fp2);
    };
    for (int mode = 0; mode < 4; ++mode) {
        const int CB = (mode & 1) ? 1 : 2;
        const bool fstream = mode >= 2;
        if (CB == 2 && s.C_out <= 32) continue;
        for (int PB = 1; PB <= 2; ++PB)
            for (int NP = 8; NP >= 2; NP >>= 1) {
                for (int NI = 2; NI <= s.N && (int64_t)NI * HoWo <= 128 * PB; ++NI) consider(CB, fstream, PB, NP, NI, 1);
                for (int tiles_y = 1; tiles_y <= s.Ho; ++tiles_y) consider(CB, fstream, PB, NP, 1, tiles_y);
            }
    }
    return best;
}

// (the search walks a few thousand candidates: more host time than a small layer runs for)
LdsPlan plan_lds(const Conv2dShape& s, int ek, const void* x, const void* w, const void* y)
{
    thread_local PlanCache<LdsPlan> cache[kFormats];
    return cache[ek].get(s, PlanCache<LdsPlan>::low_bits(x, w, y), [&] { return search_plan(s, ek, x, w, y); });
}

template <int EK, int CB, int PB, int KSC, bool FS>
hipError_t launch_lds(const void* x, const void* w, void* y, const LdsPlan& a, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_nhwc_lds_kernel<EK, CB, PB, KSC, FS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsTotal);
    if (attr != hipSuccess) return attr;
    SW_NOTED_LAUNCH(note_kernel(EK == kElemF32   ? "mfma_f32_nhwc_lds_kernel"
                                : EK == kElemF16 ? "mfma_f16_nhwc_lds_kernel"
                                : EK == kFmtS8   ? "mfma_s8_nhwc_lds_kernel"
                                : EK == kFmtS8Q  ? "mfma_s8q_nhwc_lds_kernel"
                                                 : "mfma_bf16_nhwc_lds_kernel",
                                CB + 10 * a.P.fstream, PB, a.P.NI, a.P.TH),
                    (mfma_nhwc_lds_kernel<EK, CB, PB, KSC, FS>), dim3(a.gx, a.gy), dim3(512), a.lds, st,
                    static_cast<const unsigned char*>(x), static_cast<const unsigned char*>(w), static_cast<unsigned char*>(y), a.P);
    return hipGetLastError();
}

}  // namespace

bool mfma_nhwc_lds_supported(const void* x, const void* w, const void* y, const Conv2dShape& s, int ek)
{
    return ek >= 0 && ek <= 2 && plan_lds(s, ek, x, w, y).ok;
}

bool mfma_s8_nhwc_lds_supported(const int8_t* x, const int8_t* w, const void* y, bool requant, const Conv2dShape& s)
{
    return s.dil == 1 && plan_lds(s, requant ? kFmtS8Q : kFmtS8, x, w, y).ok;
}

// fmt: Elem, kFmtS8 or kFmtS8Q
static hipError_t launch_any(const void* x, const void* w, void* y, const Conv2dShape& s, int fmt, const Epilogue& ep, const Requant& rq,
                             hipStream_t st)
{
    LdsPlan a = plan_lds(s, fmt, x, w, y);
    if (!a.ok) return hipErrorInvalidValue;
    a.P.ep = ep;
    a.P.rq = rq;
#define SW_K(CBC, PBC, KSC, FSC)                                                                    \
    switch (fmt) {                                                                                  \
    case kElemF32: return launch_lds<kElemF32, CBC, PBC, KSC, FSC>(x, w, y, a, st);                 \
    case kElemBF16: return launch_lds<kElemBF16, CBC, PBC, KSC, FSC>(x, w, y, a, st);               \
    case kElemF16: return launch_lds<kElemF16, CBC, PBC, KSC, FSC>(x, w, y, a, st);                 \
    case kFmtS8: return launch_lds<kFmtS8, CBC, PBC, KSC, FSC>(x, w, y, a, st);                     \
    default: return launch_lds<kFmtS8Q, CBC, PBC, KSC, FSC>(x, w, y, a, st);                        \
    }
#define SW_F(CBC, PBC, KSC) \
    { if (a.P.fstream) { SW_K(CBC, PBC, KSC, true) } else { SW_K(CBC, PBC, KSC, false) } }
#define SW_L(CBC, PBC)                        \
    if (a.CB == CBC && a.PB == PBC) {         \
        if (a.P.NP == 8) SW_F(CBC, PBC, 4)    \
        if (a.P.NP == 4) SW_F(CBC, PBC, 2)    \
        SW_F(CBC, PBC, 1)                     \
    }
    SW_L(2, 2); SW_L(2, 1); SW_L(1, 2); SW_L(1, 1);
#undef SW_K
#undef SW_F
#undef SW_L
    return hipErrorInvalidValue;
}

hipError_t launch_mfma_nhwc_lds(const void* x, const void* w, void* y, const Conv2dShape& s, int ek, const Epilogue& ep, hipStream_t st)
{
    if (ek < 0 || ek > 2) return hipErrorInvalidValue;
    return launch_any(x, w, y, s, ek, ep, Requant{nullptr, nullptr, 0}, st);
}

hipError_t launch_mfma_s8_nhwc_lds(const int8_t* x, const int8_t* w, void* y, const Requant* rq, const Conv2dShape& s, hipStream_t st)
{
    return launch_any(x, w, y, s, rq ? kFmtS8Q : kFmtS8, Epilogue{nullptr, 0}, rq ? *rq : Requant{nullptr, nullptr, 0}, st);
}

}  // namespace swconv
