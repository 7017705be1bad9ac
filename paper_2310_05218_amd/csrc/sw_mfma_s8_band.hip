// Quantised 3x3 convolution from packed filters, full-width row bands (paper, sections 1.1 and 3).
// The latency-tuned variant of sw_mfma_s8_packed.hip for images no wider than 64 output pixels: a launch
// of this kind has one tile per compute unit and lasts a few microseconds, so what counts is how soon after
// the wavefront starts the first matrix instruction issues and how early the first results leave.
//
//   1. One batch of scalar loads, branch-free index arithmetic.
//   2. The band of input rows a tile needs is one contiguous run per channel (the tile spans the image's
//      width).  It is fetched with 16-byte loads, copied to LDS as it is, and byte-transposed from there into
//      the [pixel][ci] operand layout (16 LDS dword reads replace 16 global dword loads per item: a global
//      load instruction is paid per lane address, not per byte).
//   3. The workgroup's packed filters (two blocks of 32 output channels, 9 * C_in / 32 KB each) are fetched
//      once with coalesced 16-byte loads and copied to LDS; every wavefront then reads the A operands of its
//      channel block into registers while its first block multiplies.
//   4. A wavefront multiplies one block of 32 pixels at a time, the K steps alternating between two
//      accumulators (so that no matrix instruction waits for the one before it), and the 16 stores of a
//      finished block are spread between the matrix instructions of the next one: output starts to leave
//      after a quarter of the multiplications, and only one block's stores remain at the end.
#include <algorithm>
#include <type_traits>

#include "swconv_internal.h"
#include "sw_s8_perm.h"

namespace swconv {

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32;
using s8perm::wgather_tap;

constexpr int kNBW = 4;            // 32-pixel blocks per wavefront at most
constexpr int kMaxPieces = 20;     // 16-byte pieces of a channel's band (up to 304 bytes)
constexpr int kWinPx = 320;        // window pixels
constexpr int kLookAhead = 3;      // operand reads run this many steps ahead of the matrix instructions

// 16 channels x 4 pixels (one dword per channel) -> four pixels x 16 channel bytes: four 4 x 4 byte transposes of
// eight v_perm_b32 each (pairs of channels interleaved first, then pairs of pairs)
__device__ __forceinline__ void transpose_16x4(const u32* in, intx4 (&out)[4])
{
    u32 o[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const u32 r0 = in[4 * g], r1 = in[4 * g + 1], r2 = in[4 * g + 2], r3 = in[4 * g + 3];
        const u32 t0 = s8perm::perm(r1, r0, 0x05010400u), t1 = s8perm::perm(r1, r0, 0x07030602u);   // (r0.b, r1.b) pairs
        const u32 u0 = s8perm::perm(r3, r2, 0x05010400u), u1 = s8perm::perm(r3, r2, 0x07030602u);
        o[0][g] = s8perm::perm(u0, t0, 0x05040100u);
        o[1][g] = s8perm::perm(u0, t0, 0x07060302u);
        o[2][g] = s8perm::perm(u1, t1, 0x05040100u);
        o[3][g] = s8perm::perm(u1, t1, 0x07060302u);
    }
#pragma unroll
    for (int px = 0; px < 4; ++px) out[px] = intx4{(int)o[px][0], (int)o[px][1], (int)o[px][2], (int)o[px][3]};
}

// n / d without a branch: magic = ceil(2^32 / d) for d > 1; d == 1 has magic 0 and one 1.  Exact while n * d < 2^32.
struct Div {
    uint32_t d, magic, one;
};
inline Div make_div(int d) { return Div{(uint32_t)d, d == 1 ? 0u : (uint32_t)(0x100000000ULL / (uint32_t)d) + 1u, d == 1 ? 1u : 0u}; }
__device__ __forceinline__ int div_by(int n, const Div& f) { return (int)(__umulhi((uint32_t)n, f.magic) + (uint32_t)n * f.one); }

struct BandParams {
    int C_out, H, W, pad, Ho, Wo, base, rem, max_pieces, wide_store;    // tile t: base + (t < rem) blocks of 32 pixels
    Div by_pieces, by_W4, by_IW, by_Wo;
};

// KS: C_in / 32.  RQ: 0 = the sums leave as int32 (y); otherwise requantised to int8 (y8): 1 = stored from the
// registers as the matrix instruction leaves them (any output size and alignment), 2 = through LDS (planes of a
// multiple of 16 pixels, y8 16-byte aligned): each wavefront requantises a finished block between the matrix
// instructions of the next one -- per value an integer add, a conversion, the product, one v_med3_f32 for both
// clamps and one fp32 add of 1.5 * 2^23, which rounds to nearest even and leaves the integer's low byte in the low
// byte of the bit pattern (clamping before rounding changes nothing: the bounds are integers and rounding is
// monotone) --, transposes 4 pixels x 4 channels inside each quad of lanes (three DPP moves, three byte permutes),
// collects its 32 channels x up to 128 pixels in its own LDS area and writes them as 16-byte pieces at the end.
//
// LDS: the window as [16-channel group][pixel][16 bytes] (group pitch = 16 mod 256 bytes, so that the staging
// writes of neighbouring groups fall into different banks; an operand read takes 16 consecutive pixels of one
// group, 256 contiguous bytes), the workgroup's packed filters as they are, and a private area per wavefront for
// the raw band of the channel groups it stages: a wavefront transposes only what it fetched itself, so the only
// workgroup barrier of the prologue is the one before the first matrix instruction.
// RAWW: wp is the filter tensor as the caller has it ([C_out][C_in][3][3]): every workgroup byte-transposes the
// filters of its 64 output channels into the packed order on their way into LDS (C_in a multiple of 64).
// NWV: wavefronts per workgroup, 4 or 8: the first four stage and multiply, the others only help with the staging
// (the byte transposes are chains of LDS reads, permutes and LDS writes: two wavefronts per SIMD overlap them).
template <int KS, int RQ, bool RAWW, int NWV>
__global__ __launch_bounds__(NWV * 64, 1) void mfma_s8_band_kernel(const int8_t* __restrict__ x, const int8_t* __restrict__ wp,
                                                              int32_t* __restrict__ y, const BandParams P,
                                                              int8_t* __restrict__ y8, const Requant rq)
{
    constexpr int C_in = 32 * KS;
    constexpr int NG = 2 * KS;                              // groups of 16 input channels
    constexpr int GP = kWinPx * 16 + 16;                    // bytes per group in the window
    constexpr int NSTEP = 9 * KS;
    static_assert(NWV == 4 || (NWV == 8 && KS == 4 && RQ != 1), "helper wavefronts exist for C_in == 128 only");
    constexpr int GPW = NG > NWV ? NG / NWV : 1;            // channel groups a wavefront stages
    constexpr int XPW = (16 * GPW * kMaxPieces + 63) / 64;  // raw 16-byte pieces per lane
    constexpr int QPW = GPW == 2 ? 32 : 64;                 // column quads per pass of a wavefront
    constexpr int XIW = (kWinPx / 4 + QPW - 1) / QPW;       // transposition passes
    static_assert(!RAWW || KS % 2 == 0, "raw filters come in chunks of 64 input channels");
    constexpr bool OWN = KS >= 2 && !RAWW;   // a wavefront keeps the half of its A operands it fetched itself in registers
    constexpr int AH = (NSTEP + 1) / 2; // A operands a wavefront fetches: the steps of its own parity
    const int C_out = P.C_out, H = P.H, W = P.W, pad = P.pad, Ho = P.Ho, Wo = P.Wo;
    constexpr int rawpitch = 16 * kMaxPieces;               // bytes per channel in the raw band (immediate offsets)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* lx = smem;                                   // [channel group][window pixel][16]
    unsigned char* la = smem + NG * GP;                         // [channel block][step][lane][16]: as packed
    unsigned char* lraw = la + 2 * NSTEP * 1024;                // per wavefront: [channel][band bytes], as in memory
    unsigned char* lrq = lraw + NWV * (16 * (NG > NWV ? NG / NWV : 1) * 16 * kMaxPieces + 144);   // (RQ == 2) [64] scales, [64] biases

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;      // K half and row/column inside a 32 x 32 block
    const int wm = (wave >> 1) & 1, wn = wave & 1;   // (of the multiplying wavefronts 0..3)
    const bool multiplier = wave < 4;
    const int n = blockIdx.y, mb = blockIdx.z;

    // the tile: blocks [blk0, blk0 + nblk) of 32 consecutive pixels of the image in row-major order, i.e. output
    // rows row0 .. row_last (the first and the last one possibly in part); its stores are whole 128-byte runs
    const int blk0 = blockIdx.x * P.base + min((int)blockIdx.x, P.rem), nblk = P.base + ((int)blockIdx.x < P.rem ? 1 : 0);
    const int HoWo = Ho * Wo;
    const int p0 = 32 * blk0, tile_px = min(32 * nblk, HoWo - p0);
    const int row0 = div_by(p0, P.by_Wo), row_last = div_by(p0 + tile_px - 1, P.by_Wo);
    const int IH = row_last - row0 + 3, IW = Wo + 2;
    const int HW = H * W;
    const int8_t* xn = x + (int64_t)n * C_in * HW;

    // ---- the padding: window cells outside the image are zeroed once (nothing else writes them)
    {
        const int cells = IH * IW;
        for (int i = tid; i < cells; i += NWV * 64) {
            const int e = div_by(i, P.by_IW), c = i - e * IW;
            const int gr = row0 - pad + e, gc = c - pad;
            if (gr < 0 || gr >= H || gc < 0 || gc >= W) {
#pragma unroll
                for (int g = 0; g < NG; ++g) *reinterpret_cast<intx4*>(lx + g * GP + i * 16) = intx4{0, 0, 0, 0};
            }
        }
    }
    // ---- the band: image rows [r_lo, r_hi) of every channel, fetched from the 16-byte boundary below its start;
    //      this wavefront takes the channels of groups g0 .. g0 + GPW - 1
    const int r_lo = max(row0 - pad, 0), r_hi = min(row0 - pad + IH, H);
    const int band_off = r_lo * W, skew = band_off & 15;
    const int npieces = (skew + (r_hi - r_lo) * W + 15) >> 4;
    const int g0 = wave * GPW;
    const bool stager = g0 < NG;                              // (C_in == 32: two groups, wavefronts 2 and 3 stage nothing)
    unsigned char* lraw_w = lraw + wave * (16 * GPW * rawpitch + 144);
    intx4 xr[XPW];
    int xraw[XPW];
#pragma unroll
    for (int k = 0; k < XPW; ++k) {
        const int idx = lane + 64 * k;
        const int cl = div_by(idx, P.by_pieces);
        const int piece = idx - cl * P.max_pieces;
        const bool ok = stager && cl < 16 * GPW && piece < npieces;
        xraw[k] = ok ? cl * rawpitch + 128 * (cl >> 4) + 16 * piece : 16 * GPW * rawpitch + 128;   // (else: a spare slot)
        const int8_t* src = xn + (ok ? (16 * g0 + cl) * HW + (band_off - skew) + 16 * piece : 0);
        xr[k] = *reinterpret_cast<const intx4*>(src);
    }
    // ---- A operands: wavefront (wm, wn) fetches the steps of parity wn of channel block wm (coalesced 16-byte loads
    //      in the packed order); issue slot k of the main loop multiplies step k ^ wn, so a[even] are these
    const intx4* wa = reinterpret_cast<const intx4*>(wp) + ((int64_t)(2 * mb + wm) * NSTEP) * 64 + lane;
    intx4 a[NSTEP];
    intx4 a_tmp[OWN || RAWW ? 1 : AH];
    // (raw filters) thread = (output channel wco of the workgroup's 64, quarter wq of a 64-channel chunk): its 16
    // channels x 9 taps are 144 contiguous bytes of the filter tensor; sixteen consecutive lanes take sixteen
    // consecutive output channels, which puts their transposed 16-byte pieces into sixteen different LDS banks
    constexpr int NCH = RAWW ? KS / 2 : 1;                 // chunks of 64 input channels
    constexpr int CPT = NCH * 4 / NWV > 0 ? NCH * 4 / NWV : 1;  // ... per thread (chunk (wave / 4) + j * NWV / 4)
    const int wco = 16 * (wave & 3) + (lane & 15), wq = lane >> 4;
    intx4 wraw[RAWW ? CPT : 1][RAWW ? 9 : 1];
    if constexpr (RAWW) {
        const int8_t* src = wp + ((int64_t)((mb << 6) + wco) * C_in + 16 * wq) * 9;
#pragma unroll
        for (int j = 0; j < CPT; ++j)
#pragma unroll
            for (int i = 0; i < 9; ++i)
                wraw[j][i] = *reinterpret_cast<const intx4*>(src + ((wave >> 2) + j * (NWV / 4)) * 576 + 16 * i);
    } else if (multiplier) {
#pragma unroll
        for (int j = 0; j < AH; ++j) {
            const int st = min(2 * j + wn, NSTEP - 1);
            if constexpr (OWN) a[2 * j] = wa[st * 64];
            else a_tmp[j] = wa[st * 64];
        }
    }

    // (RQ == 2) the workgroup's 64 scales and biases, requested behind the operands and parked in LDS with them
    float rq_scale_in = 0.0f;
    int rq_bias_in = 0;
    if constexpr (RQ == 2) {
        rq_scale_in = rq.scale[(mb << 6) + lane];
        rq_bias_in = (rq.bias ? rq.bias : reinterpret_cast<const int*>(rq.scale))[(mb << 6) + lane];
        if (!rq.bias) rq_bias_in = 0;
    }

    // ---- band -> this wavefront's LDS area as it is, then -> [group][pixel][16] with the byte transposes:
    //      item = (channel group, column quad of a window row); LDS operations of a wavefront complete in order
#pragma unroll
    for (int k = 0; k < XPW; ++k)
        *reinterpret_cast<intx4*>(lraw_w + xraw[k]) = xr[k];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (stager) {
        const int W4 = W >> 2;
        const int nquads = IH * W4;
        const int gl = GPW == 2 ? (lane & 1) : 0;
        const int qslot = GPW == 2 ? (lane >> 1) : lane;
#pragma unroll
        for (int k = 0; k < XIW; ++k) {
            const int quad = qslot + QPW * k;
            const int e = div_by(quad, P.by_W4);
            const int cq = quad - e * W4;
            const int r = row0 - pad + e;
            if (quad < nquads && r >= r_lo && r < r_hi) {
                const unsigned char* src = lraw_w + gl * (16 * rawpitch + 128) + skew + (r - r_lo) * W + 4 * cq;
                u32 v[16];
#pragma unroll
                for (int c = 0; c < 16; ++c) v[c] = *reinterpret_cast<const u32*>(src + c * rawpitch);
                unsigned char* dst = lx + (g0 + gl) * GP + (e * IW + pad + 4 * cq) * 16;
                intx4 t[4];
                transpose_16x4(v, t);
                *reinterpret_cast<intx4*>(dst) = t[0];
                *reinterpret_cast<intx4*>(dst + 16) = t[1];
                *reinterpret_cast<intx4*>(dst + 32) = t[2];
                *reinterpret_cast<intx4*>(dst + 48) = t[3];
            }
        }
    }
    if constexpr (RQ == 2) {
        if (wave == 0) {
            reinterpret_cast<float*>(lrq)[lane] = rq_scale_in;
            reinterpret_cast<int*>(lrq + 256)[lane] = rq_bias_in;
        }
    }
    // ---- the fetched A operands -> LDS, for the partner wavefront (and, for C_in == 32, for this one as well)
    if constexpr (RAWW) {
        // channel block wco / 32, step = tap * KS + 2 * chunk + wq / 2, operand lane = wco % 32 + 32 * (wq % 2)
        unsigned char* dst = la + (((wco >> 5) * NSTEP + (wq >> 1)) * 64 + (wco & 31) + 32 * (wq & 1)) * 16;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            u32 raw[36];
#pragma unroll
            for (int i = 0; i < 9; ++i) {
                raw[4 * i + 0] = (u32)wraw[j][i].x; raw[4 * i + 1] = (u32)wraw[j][i].y;
                raw[4 * i + 2] = (u32)wraw[j][i].z; raw[4 * i + 3] = (u32)wraw[j][i].w;
            }
            unsigned char* d = dst + 2 * ((wave >> 2) + j * (NWV / 4)) * 1024;
            *reinterpret_cast<intx4*>(d + 0 * KS * 1024) = wgather_tap<0>(raw);
            *reinterpret_cast<intx4*>(d + 1 * KS * 1024) = wgather_tap<1>(raw);
            *reinterpret_cast<intx4*>(d + 2 * KS * 1024) = wgather_tap<2>(raw);
            *reinterpret_cast<intx4*>(d + 3 * KS * 1024) = wgather_tap<3>(raw);
            *reinterpret_cast<intx4*>(d + 4 * KS * 1024) = wgather_tap<4>(raw);
            *reinterpret_cast<intx4*>(d + 5 * KS * 1024) = wgather_tap<5>(raw);
            *reinterpret_cast<intx4*>(d + 6 * KS * 1024) = wgather_tap<6>(raw);
            *reinterpret_cast<intx4*>(d + 7 * KS * 1024) = wgather_tap<7>(raw);
            *reinterpret_cast<intx4*>(d + 8 * KS * 1024) = wgather_tap<8>(raw);
        }
    } else if (multiplier) {
        unsigned char* la_own = la + (wm * NSTEP * 64 + lane) * 16;
#pragma unroll
        for (int j = 0; j < AH; ++j) {
            const int st = 2 * j + wn;
            if (st < NSTEP) {
                if constexpr (OWN) *reinterpret_cast<intx4*>(la_own + st * 1024) = a[2 * j];
                else *reinterpret_cast<intx4*>(la_own + st * 1024) = a_tmp[j];
            }
        }
    }
    __syncthreads();
    if (!multiplier) return;

    // the tile's blocks in two halves, one per wavefront pair member
    const int half = (nblk + 1) >> 1;
    const int first = wn * half;
    const int live = __builtin_amdgcn_readfirstlane(wn == 0 ? half : nblk - half);
    if (live == 0) return;

    const int co_base = (mb << 6) + 32 * wm + 4 * lg;       // this lane's first output channel
    const int64_t ybase = ((int64_t)n * C_out + co_base) * HoWo;
    const int rowoff1 = IW * 16, rowoff2 = 2 * IW * 16;
    // issue slot k multiplies K step (OWN ? k ^ wn : k): its A operand (odd slots, or all of them) in LDS and the
    // channel group of its B operand
    const unsigned char* la_w = la + (wm * NSTEP * 64 + lane) * 16 + (OWN ? (1 - wn) * 1024 - 1024 : 0);
    const int gsel_even = OWN ? 2 * wn + lg : lg, gsel_odd = OWN ? 2 * (1 - wn) + lg : lg;

    // this lane's sixteen output channels' scales and biases, read once
    float rq_scale[RQ == 1 ? 16 : 1];
    int rq_bias[RQ == 1 ? 16 : 1];
    if constexpr (RQ == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int co = co_base + 8 * (v >> 2) + (v & 3);
            rq_scale[v] = rq.scale[co];
            rq_bias[v] = rq.bias ? rq.bias[co] : 0;
        }
    }
    auto requant_reg = [&](int acc_v, int v) __attribute__((always_inline)) {
        float r = rintf(__int2float_rn(acc_v + rq_bias[RQ == 1 ? v : 0]) * rq_scale[RQ == 1 ? v : 0]);
        r = fminf(fmaxf(r, rq.relu ? 0.0f : -128.0f), 127.0f);
        return (int)r;
    };
    // Requantised output, rows whose groups of four pixels are aligned dwords in y8 (P.wide_store): the four
    // lanes of a quad hold four pixels x four consecutive channels; two exchange rounds inside the quad
    // (DPP quad_perm) transpose that, so that lane k ends up with channel k of all four pixels and stores
    // them as one dword instead of four single bytes.
    auto store_quad = [&](int dst, const intx16& c, int g) __attribute__((always_inline)) {
        const int k = lane & 3;
        int r[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) r[t] = requant_reg(c[4 * g + t], 4 * g + t) & 255;
        const bool b0 = k & 1, b1 = k & 2;
        const int keep01 = b0 ? r[1] : r[0], send01 = b0 ? r[0] : r[1];
        const int keep23 = b0 ? r[3] : r[2], send23 = b0 ? r[2] : r[3];
        const int got01 = __builtin_amdgcn_mov_dpp(send01, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
        const int got23 = __builtin_amdgcn_mov_dpp(send23, 0xB1, 0xF, 0xF, true);
        const int own_a = b1 ? keep23 : keep01, own_b = b1 ? got23 : got01;
        const int snd_a = b1 ? keep01 : keep23, snd_b = b1 ? got01 : got23;
        const int far_a = __builtin_amdgcn_mov_dpp(snd_a, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
        const int far_b = __builtin_amdgcn_mov_dpp(snd_b, 0x4E, 0xF, 0xF, true);
        // channel k of pixels k (own_a), k^1 (own_b), k^2 (far_a), k^3 (far_b); byte j of the dword is pixel j
        const unsigned word = (unsigned)own_a << (8 * k) | (unsigned)own_b << (8 * (k ^ 1)) |
                              (unsigned)far_a << (8 * (k ^ 2)) | (unsigned)far_b << (8 * (k ^ 3));
        if (dst >= 0)
            *reinterpret_cast<unsigned*>(y8 + ybase + (int64_t)(8 * g + k) * HoWo + (dst - k)) = word;
    };
    auto store_reg = [&](int dst, const intx16& c, int v) __attribute__((always_inline)) {
        const int ch = 8 * (v >> 2) + (v & 3);
        if constexpr (RQ) {
            if (P.wide_store) {
                if ((v & 3) == 3) store_quad(dst, c, v >> 2);
            } else if (dst >= 0) {
                y8[ybase + (int64_t)ch * HoWo + dst] = (int8_t)requant_reg(c[v], v);
            }
        } else {
            if (dst >= 0) __builtin_nontemporal_store(c[v], y + ybase + (int64_t)ch * HoWo + dst);
        }
    };

    // (RQ == 2) the requantisation of one block in 32 micro-steps, eight per group g of four registers (channels
    // 8g + 4lg + 0..3 of this lane's pixel): four values, the packing, the exchange inside the quad, the byte
    // selection, the LDS write.  Lane k of a quad ends up with channel 8g + 4lg + k of the quad's four pixels.
    constexpr int kOutPitch = 160;                            // bytes per channel in the output area (bank-conflict-free)
    unsigned char* lout = lraw_w;                             // (the raw band is dead after the prologue)
    const int qk = lane & 3;
    const u32 sel_own = 0x0c0c0c0cu ^ ((0x0cu ^ (u32)qk) << (8 * qk)) ^ ((0x0cu ^ (u32)(4 + qk)) << (8 * (qk ^ 1)));
    const u32 sel_far = 0x0c0c0c0cu ^ ((0x0cu ^ (u32)qk) << (8 * (qk ^ 2))) ^ ((0x0cu ^ (u32)(4 + qk)) << (8 * (qk ^ 3)));
    const float rq_lo = rq.relu ? 0.0f : -128.0f;
    u32 rqv[4], rq_packed = 0, rq_a = 0, rq_b = 0, rq_c = 0, rq_word = 0;
    // scales and biases of the group's four channels come from LDS one group ahead (they would cost 32 registers)
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    const unsigned char* lrq_lane = lrq + (32 * wm + 4 * lg) * 4;
    floatx4 rq_sc = *reinterpret_cast<const floatx4*>(lrq_lane);
    intx4 rq_bi = *reinterpret_cast<const intx4*>(lrq_lane + 256);
    unsigned char* lout_lane = lout + (4 * lg + qk) * kOutPitch + 4 * (lj >> 2);
    auto rq_step = [&](int ms, const intx16& c, int blk) __attribute__((always_inline)) {
        const int g = ms >> 3, t = ms & 7;
        if (t < 4) {
            const int v = 4 * g + t;
            float f = __int2float_rn(c[v] + rq_bi[t]) * rq_sc[t];
            f = __builtin_amdgcn_fmed3f(f, rq_lo, 127.0f);
            rqv[t] = __float_as_uint(f + 12582912.0f);
        } else if (t == 4) {
            rq_packed = s8perm::perm(s8perm::perm(rqv[3], rqv[2], 0x04000c0cu), s8perm::perm(rqv[1], rqv[0], 0x0c0c0400u), 0x07060100u);
        } else if (t == 5) {
            rq_a = (u32)__builtin_amdgcn_mov_dpp((int)rq_packed, 0xB1, 0xF, 0xF, true);   // from lane k ^ 1
            rq_b = (u32)__builtin_amdgcn_mov_dpp((int)rq_packed, 0x4E, 0xF, 0xF, true);   // k ^ 2
            rq_c = (u32)__builtin_amdgcn_mov_dpp((int)rq_packed, 0x1B, 0xF, 0xF, true);   // k ^ 3
        } else if (t == 6) {
            rq_word = s8perm::perm(rq_a, rq_packed, sel_own) | s8perm::perm(rq_c, rq_b, sel_far);
            rq_sc = *reinterpret_cast<const floatx4*>(lrq_lane + 32 * ((g + 1) & 3));
            rq_bi = *reinterpret_cast<const intx4*>(lrq_lane + 256 + 32 * ((g + 1) & 3));
        } else {
            *reinterpret_cast<u32*>(lout_lane + 8 * g * kOutPitch + 32 * blk) = rq_word;
        }
    };

    // One block of 32 pixels: all K steps, even issue slots into one accumulator and odd ones into the other (so that
    // no matrix instruction waits for the one before it).  FIRST: the A operands that are not in registers yet come
    // from LDS on the way (and stay in registers); DRAIN: the 16 stores of the block before (prev at offset
    // prev_dst) are spread between the matrix instructions.
    auto block = [&](auto first_tag, auto drain_tag, int i, const intx16& prev, int prev_dst) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value, DRAIN = decltype(drain_tag)::value;
        int p = (first + i) * 32 + lj;
        if (p >= tile_px) p = 0;
        const int pi = div_by(p0 + p, P.by_Wo), pj = p0 + p - pi * Wo;
        const int cell = (pi - row0) * IW + pj;
        const unsigned char* bb_even = lx + gsel_even * GP + cell * 16;
        const unsigned char* bb_odd = lx + gsel_odd * GP + cell * 16;
        auto b_at = [&](int k) __attribute__((always_inline)) {
            // slot k: step k ^ wn (or k): tap = step / KS is the same for both, the K quarter's upper bits as well
            const int tap = k / KS;
            const int r = tap / 3, q = tap - 3 * r;
            const int kk_hi = OWN ? ((k % KS) & ~1) : (k % KS);       // (its lowest bit is in the base pointer)
            const unsigned char* base = (k & 1) ? bb_odd : bb_even;
            return *reinterpret_cast<const intx4*>(base + 2 * kk_hi * GP + (r == 0 ? 0 : r == 1 ? rowoff1 : rowoff2) + q * 16);
        };
        auto a_from_lds = [&](int k) __attribute__((always_inline)) {
            if (FIRST && (!OWN || (k & 1))) a[k] = *reinterpret_cast<const intx4*>(la_w + k * 1024);
        };
        intx16 acc0, acc1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc0[v] = 0; acc1[v] = 0; }
        intx4 b[kLookAhead + 1];
#pragma unroll
        for (int k = 0; k < kLookAhead && k < NSTEP; ++k) {
            a_from_lds(k);
            b[k] = b_at(k);
        }
        // 16 stores over the steps (KS == 1: two per step over the first eight)
        constexpr int PER = NSTEP >= 18 ? 1 : 2;
        constexpr int GAP = NSTEP >= 34 ? 2 : 1;
#pragma unroll
        for (int k = 0; k < NSTEP; ++k) {
            if (k + kLookAhead < NSTEP) {
                a_from_lds(k + kLookAhead);
                b[(k + kLookAhead) % (kLookAhead + 1)] = b_at(k + kLookAhead);
            }
            if constexpr (RQ == 2) {
                if (DRAIN) {
                    constexpr int MPER = (32 + NSTEP - 1) / NSTEP;    // micro-steps per issue slot
#pragma unroll
                    for (int u = 0; u < MPER; ++u)
                        if (k * MPER + u < 32) rq_step(k * MPER + u, prev, i - 1);
                }
            } else if (DRAIN && k % GAP == 0) {
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int sv = (k / GAP) * PER + u;
                    if (sv < 16) store_reg(prev_dst, prev, sv);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (k & 1) acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[k], b[k % (kLookAhead + 1)], acc1, 0, 0, 0);
            else acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[k], b[k % (kLookAhead + 1)], acc0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        intx16 out;
#pragma unroll
        for (int v = 0; v < 16; ++v) out[v] = acc0[v] + acc1[v];
        return out;
    };
    // offset of this lane's pixel in block i inside a channel plane (-1 when it lies outside the tile/image)
    auto block_dst = [&](int i) -> int {
        const int p = (first + i) * 32 + lj;
        return p < tile_px ? p0 + p : -1;
    };

    intx16 res = block(std::true_type{}, std::false_type{}, 0, intx16{}, -1);
    int dst = block_dst(0);
#pragma unroll 1
    for (int i = 1; i < live; ++i) {
        const intx16 nxt = block(std::false_type{}, std::true_type{}, i, res, dst);
        res = nxt;
        dst = block_dst(i);
    }
    if constexpr (RQ == 2) {
#pragma unroll
        for (int ms = 0; ms < 32; ++ms) rq_step(ms, res, live - 1);
        // this wavefront's 32 channels x vbytes pixels leave as 16-byte pieces (eight slots per channel)
        const int vbytes = min(32 * live, tile_px - 32 * first);
        int8_t* yo = y8 + ((int64_t)n * C_out + (mb << 6) + 32 * wm) * HoWo + p0 + 32 * first;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = lane + 64 * j, ch = e >> 3, part = e & 7;
            const intx4 v = *reinterpret_cast<const intx4*>(lout + ch * kOutPitch + 16 * part);
            if (16 * part < vbytes) __builtin_nontemporal_store(v, reinterpret_cast<intx4*>(yo + (int64_t)ch * HoWo + 16 * part));
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) store_reg(dst, res, v);
    }
}

struct BandTiling {
    int base, rem, tiles, max_pieces;
    bool ok;
};

// Tiles of up to 2 * kNBW blocks of 32 consecutive pixels (row-major over the image, so that every store covers
// whole 128-byte runs of the output whatever the image width), evenly sized; the rows a tile touches plus the
// filter halo must fit kWinPx window pixels and kMaxPieces 16-byte pieces per channel.
BandTiling pick_band(const Conv2dShape& s)
{
    BandTiling t{0, 0, 0, 0, false};
    if (s.Wo > 64) return t;
    const int HoWo = s.Ho * s.Wo, blocks = (HoWo + 31) / 32;
    for (int nb = 2 * kNBW; nb >= 1 && !t.ok; --nb) {
        const int tiles = (blocks + nb - 1) / nb, base = blocks / tiles, rem = blocks % tiles;
        bool fits = true;
        int max_pieces = 1;
        for (int i = 0; i < tiles && fits; ++i) {
            const int p0 = 32 * (i * base + std::min(i, rem)), px = std::min(32 * (base + (i < rem ? 1 : 0)), HoWo - p0);
            const int row0 = p0 / s.Wo, row_last = (p0 + px - 1) / s.Wo, IH = row_last - row0 + 3;
            const int r_lo = std::max(row0 - s.pad, 0), r_hi = std::min(row0 - s.pad + IH, s.H);
            const int pieces = (((r_lo * s.W) & 15) + (r_hi - r_lo) * s.W + 15) / 16;
            fits = IH * (s.Wo + 2) <= kWinPx && pieces <= kMaxPieces && r_hi > r_lo;
            max_pieces = std::max(max_pieces, pieces);
        }
        if (fits) t = BandTiling{base, rem, tiles, max_pieces, true};
    }
    t.ok = t.ok && s.N <= 65535 && s.C_out / 64 <= 65535;
    return t;
}

template <int KS, int RQ, bool RAWW>
hipError_t launch_band(const int8_t* x, const int8_t* wp, int32_t* y, int8_t* y8, const Requant& rq, const Conv2dShape& s,
                       const BandTiling& t, hipStream_t st)
{
    // helper wavefronts where the register budget allows two wavefronts per SIMD (the requantising stores need more)
    constexpr int NWV = (KS == 4 && RQ != 1) ? 8 : 4;
    constexpr int GPW = 2 * KS > NWV ? 2 * KS / NWV : 1;     // as in the kernel
    constexpr int kLds = 2 * KS * (kWinPx * 16 + 16) + 2 * 9 * KS * 1024 + NWV * (16 * GPW * 16 * kMaxPieces + 144) + (RQ == 2 ? 512 : 0);
    const size_t lds = kLds;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_s8_band_kernel<KS, RQ, RAWW, NWV>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                                       kLds);
    if (attr != hipSuccess) return attr;
    BandParams P;
    P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo; P.base = t.base; P.rem = t.rem;
    P.max_pieces = t.max_pieces;
    // (requantised output only) dword stores of four pixels: groups of four pixels must be aligned dwords of y8
    P.wide_store = (s.Ho * s.Wo) % 4 == 0 && reinterpret_cast<uintptr_t>(y8) % 4 == 0;
    P.by_pieces = make_div(t.max_pieces);
    P.by_W4 = make_div(s.W / 4);
    P.by_IW = make_div(s.Wo + 2);
    P.by_Wo = make_div(s.Wo);
    note_kernel("mfma_s8_band_kernel", KS, RQ, RAWW);
    hipLaunchKernelGGL((mfma_s8_band_kernel<KS, RQ, RAWW, NWV>), dim3((unsigned)t.tiles, (unsigned)s.N, (unsigned)(s.C_out / 64)),
                       dim3(NWV * 64), lds, st, x, wp, y, P, y8, rq);
    return hipGetLastError();
}

}  // namespace

// raw_filters: w is the caller's [C_out][C_in][3][3] tensor (C_in a multiple of 64), else the packed copy.
bool mfma_s8_band_supported(const int8_t* x, const int8_t* w, const Conv2dShape& s, bool raw_filters)
{
    if (s.stride != 1 || s.R != 3 || s.S != 3 || s.dil != 1) return false;
    if (s.C_in != 32 && s.C_in != 64 && s.C_in != 128) return false;
    if (raw_filters && s.C_in % 64 != 0) return false;
    if (s.C_out % 64 != 0 || s.W % 4 != 0 || ((int64_t)s.H * s.W) % 16 != 0) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || reinterpret_cast<uintptr_t>(w) % 16 != 0) return false;
    return pick_band(s).ok;
}

hipError_t launch_mfma_s8_band(const int8_t* x, const int8_t* w, int32_t* y, int8_t* y8, const Requant* rq,
                               const Conv2dShape& s, bool raw_filters, hipStream_t st)
{
    const BandTiling t = pick_band(s);
    const Requant none{nullptr, nullptr, 0};
    const int KS = s.C_in / 32;
    // requantised output through LDS: 16-byte pieces of y8 must be aligned and never straddle the end of a plane
    const bool staged = rq && (s.Ho * s.Wo) % 16 == 0 && reinterpret_cast<uintptr_t>(y8) % 16 == 0;
#define SW_BAND(KSC, RAWC)                                                                   \
    do {                                                                                     \
        if (rq && staged) return launch_band<KSC, 2, RAWC>(x, w, nullptr, y8, *rq, s, t, st); \
        if (rq) return launch_band<KSC, 1, RAWC>(x, w, nullptr, y8, *rq, s, t, st);          \
        return launch_band<KSC, 0, RAWC>(x, w, y, nullptr, none, s, t, st);                  \
    } while (0)
    if (raw_filters) {
        if (KS == 4) SW_BAND(4, true);
        SW_BAND(2, true);
    }
    if (KS == 4) SW_BAND(4, false);
    if (KS == 2) SW_BAND(2, false);
    SW_BAND(1, false);
#undef SW_BAND
}

}  // namespace swconv
