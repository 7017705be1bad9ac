// The multi-channel fp32 sliding sum for filters of few taps (1x1 ... 4x4; any stride, padding and dilation; C_in a
// multiple of 8) with both operands brought into LDS by direct-to-LDS buffer loads: no staging registers, no
// transposition, the next chunk of channels in flight while this one multiplies (paper, section 3: every tap a small
// matrix product; section 2: the input is used as it lies in memory, padding included).
//
//   x [N, C_in, H, W]     w [C_out, C_in, R, S]     y [N, C_out, H_out, W_out]     fp32
//
// A direct-to-LDS load writes what lane l fetched to LDS address base + size * l (4 or 16 bytes per lane), whatever
// global address the lane asked for, and zeros for an address beyond the buffer.  Two layouts follow from that:
//
//   window   [channel of the chunk][cell]          one float per cell, 4-byte loads: consecutive lanes take
//            consecutive cells of the rectangle of input pixels the tile touches (cells in the padding are addresses
//            beyond the buffer: they arrive as zeros);
//   filters  [output channel][16-byte piece j]     piece j of an output channel = floats 4j .. 4j+3 of its run of
//            CK * R * S filter values (channels of the chunk, taps fastest), as they lie in w: 16-byte loads whose
//            consecutive lanes take consecutive pieces (whole cache lines of w); the row pitch is an odd number of
//            pieces (a padding piece where needed), which spreads the 32 rows of an operand read over all banks.
//
// The K index of v_mfma_f32_32x32x2_f32 is only a summation index, so it runs over e = (channel, tap) in the order of
// the filter run: step t of lane half kk in group g is e = 8g + 4kk + t.  A lane's A operands for four steps are then
// ONE 16-byte LDS read (piece 2g + kk of its output channel), and its B operands are four 4-byte reads at
// cell(pixel) + offset[e], offset[e] = channel * cells + (r * IW + s) * dilation from a table in LDS: the tap shift is
// an address, stride and dilation are factors in it, no column matrix exists.
//
// Workgroup = 64 output channels x up to 128 NBW output pixels: whole rows of one image, or several whole images when
// they are small; the pixels of a tile are numbered row-major and cut into blocks of 32, block 4b + w going to
// multiplying wavefront w of four.  Four more wavefronts only load.  Two LDS stages: after the barrier that ends chunk
// c - 1 the loaders issue chunk c + 1's loads (which need no registers) and wait for them before the next barrier,
// while the multipliers work on chunk c; operand reads run one group ahead of the matrix instructions.
#include <algorithm>
#include <type_traits>

#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

#define SW_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int kMaxNS = 10;                     // window slots of 64 cells per channel
constexpr int kMaxFI = 10;                     // filter loads per loading wavefront and chunk
constexpr size_t kLdsBudget = 80 * 1024;       // two workgroups per CU
constexpr unsigned kBeyond = 0x80000000u;      // a byte offset no tensor of less than 2 GiB reaches

struct DmaParams {
    Epilogue ep;
    int N, C_in, C_out, H, W, Ho, Wo, stride, pad, dil, S;
    int CK, RS, NG;                // channels per chunk, taps, groups of eight K values per chunk (CK * RS / 8)
    int PC, PCp;                   // 16-byte filter pieces per output channel and chunk (CK * RS / 4); the same made odd
    int NI, TH, tiles_y;           // images and output rows per tile, row tiles per image
    int IH, IW, cells_img;         // window rows and columns of one image, their product
    int WC, WCp, NS;               // cells per channel (NI * cells_img), rounded up to whole slots, slots
    int tile_px;                   // NI * TH * Wo
    int chunks;
    int stage_bytes, win_off, tbl_off;
    unsigned x_bytes, w_bytes;
    FastDiv by_tiles_y, by_cells_img, by_IW, by_thwo, by_Wo, by_RS, by_S, by_PCp;
};

// Wavefronts 0 .. 3 multiply, wavefronts 4 .. 7 only load: a wavefront that issues loads sits in their issue until the
// memory pipeline has taken them, and in a wavefront of its own that wait holds no matrix instruction back.
// NGT: the number of groups per chunk as a compile-time constant (0: run-time): the loop over groups is unrolled, the
// per-K offsets stay in registers (no table reads) and all address arithmetic of a group sits in one slot.
// BW x KS multiplying wavefronts: BW take the tile's blocks in turn (block BW b + wb), and KS wavefronts share each
// block, every KS-th group of K values each; their partial sums meet in LDS at the end.  KS > 1 is for launches of
// at most one workgroup per CU: two wavefronts per SIMD hide part of what the operand reads cost, and a tile of few
// blocks still occupies every SIMD.
template <int NBW, int NGT, int BW, int KS>
__global__ __launch_bounds__(64 * (BW * KS + 4), KS == 1 ? 4 : 3) void mfma_f32_dma_kernel(const float* __restrict__ x,
                                                                                          const float* __restrict__ w,
                                                                                          float* __restrict__ y, const DmaParams P)
{
    constexpr int MW = BW * KS;                 // multiplying wavefronts
    static_assert(NGT == 0 || KS == 1, "the unrolled group loop takes every group");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ig = fast_div(blockIdx.x, P.by_tiles_y), ty = blockIdx.x - ig * P.tiles_y;
    const int n0 = ig * P.NI, row0 = ty * P.TH;
    const int co0 = blockIdx.y * 64;

    if (wave >= MW) {
        // ---------------------------------------------------------------------------------------- the loaders
        const int lw = wave - MW;
        const int HW = P.H * P.W;
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, P.x_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(w), 0, P.w_bytes, 0x00020000);
        // this lane's cell in each window slot: byte offset of the input pixel in channel 0 of its image
        unsigned wbase[kMaxNS];
#pragma unroll
        for (int s = 0; s < kMaxNS; ++s) {
            const int cell = 64 * s + lane;
            const int i = fast_div(cell, P.by_cells_img), rem = cell - i * P.cells_img;
            const int e = fast_div(rem, P.by_IW), f = rem - e * P.IW;
            const int gr = row0 * P.stride - P.pad + e, gc = f - P.pad, n = n0 + i;
            const bool in = cell < P.WC && n < P.N && gr >= 0 && gr < P.H && gc >= 0 && gc < P.W;
            wbase[s] = in ? (unsigned)((n * P.C_in * HW + gr * P.W + gc) * 4) : kBeyond;
        }
        // this lane's 16-byte slot in each filter load of this wavefront (loads lw, lw + 4, ...): slot q of the
        // stage's filter area is piece q % PCp of output channel q / PCp; the last piece of a row may be padding
        unsigned fbase[kMaxFI];
#pragma unroll
        for (int k = 0; k < kMaxFI; ++k) {
            const int q = 64 * (lw + 4 * k) + lane;
            const int co = fast_div(q, P.by_PCp), j = q - co * P.PCp;
            fbase[k] = (j < P.PC && co < 64 && co0 + co < P.C_out) ? (unsigned)((co0 + co) * P.C_in * P.RS * 4 + 16 * j) : kBeyond;
        }
        auto issue = [&](int c, int stage) __attribute__((always_inline)) {
            unsigned char* sf = smem + stage * P.stage_bytes;
            unsigned char* sw = sf + P.win_off;
            const int ci0 = c * P.CK;
#pragma unroll 1
            for (int ci = lw; ci < P.CK; ci += 4) {
                const unsigned choff = (unsigned)((ci0 + ci) * HW * 4);
                unsigned char* dst = sw + ci * P.WCp * 4;
#pragma unroll
                for (int s = 0; s < kMaxNS; ++s)
                    if (s < P.NS) __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, SW_LDS_PTR(dst + 256 * s), 4, wbase[s] + choff, 0, 0, 0);
            }
            const unsigned foff = (unsigned)(ci0 * P.RS * 4);
#pragma unroll
            for (int k = 0; k < kMaxFI; ++k)
                if (lw + 4 * k < P.PCp)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, SW_LDS_PTR(sf + 1024 * (lw + 4 * k)), 16, fbase[k] + foff, 0, 0, 0);
        };
        issue(0, 0);
        __syncthreads();                                // (the multipliers' table)
#pragma unroll 1
        for (int c = 0; c < P.chunks; ++c) {
            __builtin_amdgcn_s_waitcnt(0);              // this wavefront's loads of chunk c have landed
            __syncthreads();                            // barrier c: chunk c is complete, chunk c - 1 has been multiplied
            if (c + 1 < P.chunks) issue(c + 1, (c + 1) & 1);
        }
        __builtin_amdgcn_s_waitcnt(0);
        if constexpr (KS > 1) {                         // (the two barriers around the partial sums)
            __syncthreads();
            __syncthreads();
        }
        return;
    }

    // -------------------------------------------------------------------------------------------- the multipliers
    const int lj = lane & 31, kk = lane >> 5;
    // byte offset of K value e = (channel, tap) from a pixel's cell
    {
        int* tbl = reinterpret_cast<int*>(smem + P.tbl_off);
        for (int e = tid; e < P.CK * P.RS; e += 64 * MW) {
            const int ci = fast_div(e, P.by_RS), tap = e - ci * P.RS;
            const int r = fast_div(tap, P.by_S), s = tap - r * P.S;
            tbl[e] = 4 * (ci * P.WCp + (r * P.IW + s) * P.dil);
        }
    }
    // this wavefront's pixel blocks: block BW b + wb of the tile
    const int HoWo = P.Ho * P.Wo;
    const int thwo = P.TH * P.Wo;
    const int valid_px = P.NI > 1 ? min(P.NI, P.N - n0) * HoWo : min(P.TH, P.Ho - row0) * P.Wo;
    // block column; part of K (the parts of a block on neighbouring wavefronts, i.e. on different SIMDs)
    const int wb = KS == 1 ? wave : wave / KS, kp = KS == 1 ? 0 : wave % KS;
    int nlive = 0;
    int pixoff[NBW];
#pragma unroll
    for (int b = 0; b < NBW; ++b) {
        const int p = 32 * (BW * b + wb) + lj;
        if (32 * (BW * b + wb) < valid_px) nlive = b + 1;
        const int i = fast_div(p, P.by_thwo), rem = p - i * thwo;
        const int ol = fast_div(rem, P.by_Wo), ow = rem - ol * P.Wo;
        pixoff[b] = p < valid_px ? 4 * (i * P.cells_img + (ol * P.IW + ow) * P.stride) : 0;
    }

    floatx16 acc[NBW][2];
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc[b][0][v] = 0.f; acc[b][1][v] = 0.f; }

    // One chunk on NL blocks.  Group g = K values 8g .. 8g + 7 = 8 NL matrix instructions; a wavefront issues in order, so
    // what keeps the matrix pipe busy is other work placed BETWEEN its instructions: behind the first one sit the
    // operand reads of group g + 1 (into the other register set) and the read of the offsets of group g + 2.
    const int arow = 16 * P.PCp;                                                // bytes per output channel's filter row
    const unsigned char* tp = smem + P.tbl_off + 16 * kk;                       // + 32 g
    __syncthreads();                                                            // (the table; the loaders pass it too)
    const int glast = kp + ((P.NG - 1 - kp) / KS) * KS;                         // this wavefront's last group (NG > kp)
    const intx4 tfirst = *reinterpret_cast<const intx4*>(tp + 32 * min(kp, glast));
    const intx4 tsecond = *reinterpret_cast<const intx4*>(tp + 32 * min(kp + KS, glast));
    auto multiply = [&](auto nl_tag, int stage) __attribute__((always_inline)) {
        constexpr int NL = decltype(nl_tag)::value;
        struct Ops {
            floatx4 a0, a1;
            float b[NL][4];
        };
        const unsigned char* sf = smem + stage * P.stage_bytes;
        const unsigned char* ap0 = sf + lj * arow + 16 * kk;                    // + 32 g
        const unsigned char* ap1 = ap0 + 32 * arow;                             // the upper 32 channels
        const unsigned char* bp = sf + P.win_off;
        auto group = [&](const Ops& cur, Ops& nxt, const intx4& tn, intx4& tl, int g) __attribute__((always_inline)) {
            const int gn = min(g + KS, glast), g2 = min(g + 2 * KS, glast);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int b = 0; b < NL; ++b)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int m = (t * NL + b) * 2 + h;
                        acc[b][h] = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? cur.a1[t] : cur.a0[t], cur.b[b][t], acc[b][h], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        // everything else of the group in ONE slot: a matrix instruction that follows another issues
                        // without a gap, one that follows anything else pays a few cycles, however much else it was
                        if (m == 0) {
                            nxt.a0 = *reinterpret_cast<const floatx4*>(ap0 + 32 * gn);
                            nxt.a1 = *reinterpret_cast<const floatx4*>(ap1 + 32 * gn);
#pragma unroll
                            for (int bq = 0; bq < NL; ++bq)
#pragma unroll
                                for (int tq = 0; tq < 4; ++tq) nxt.b[bq][tq] = *reinterpret_cast<const float*>(bp + pixoff[bq] + tn[tq]);
                            tl = *reinterpret_cast<const intx4*>(tp + 32 * g2);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
        };
        Ops X, Y;
        X.a0 = *reinterpret_cast<const floatx4*>(ap0 + 32 * kp);
        X.a1 = *reinterpret_cast<const floatx4*>(ap1 + 32 * kp);
#pragma unroll
        for (int b = 0; b < NL; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) X.b[b][t] = *reinterpret_cast<const float*>(bp + pixoff[b] + tfirst[t]);
        intx4 ta = tsecond, tb = tsecond;
#pragma unroll 1
        for (int g = kp; g < P.NG; g += 2 * KS) {
            group(X, Y, ta, tb, g);
            if (g + KS < P.NG) group(Y, X, tb, ta, g + KS);
        }
    };

    // The same with the group loop unrolled and the offsets of every K value in registers (no table reads).
    int treg[NGT > 0 ? NGT : 1][4];
    if constexpr (NGT > 0) {
#pragma unroll
        for (int g = 0; g < NGT; ++g) {
            const intx4 t = *reinterpret_cast<const intx4*>(tp + 32 * g);
            treg[g][0] = t[0]; treg[g][1] = t[1]; treg[g][2] = t[2]; treg[g][3] = t[3];
        }
    }
    auto multiply_unrolled = [&](int stage) __attribute__((always_inline)) {
        constexpr int NL = NBW;
        struct Ops {
            floatx4 a0, a1;
            float b[NL][4];
        };
        const unsigned char* sf = smem + stage * P.stage_bytes;
        const unsigned char* ap0 = sf + lj * arow + 16 * kk;
        const unsigned char* ap1 = ap0 + 32 * arow;
        const unsigned char* bb[NL];
#pragma unroll
        for (int b = 0; b < NL; ++b) bb[b] = sf + P.win_off + pixoff[b];
        Ops ops[2];
        ops[0].a0 = *reinterpret_cast<const floatx4*>(ap0);
        ops[0].a1 = *reinterpret_cast<const floatx4*>(ap1);
#pragma unroll
        for (int b = 0; b < NL; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) ops[0].b[b][t] = *reinterpret_cast<const float*>(bb[b] + treg[0][t]);
#pragma unroll
        for (int g = 0; g < NGT; ++g) {
            const Ops& cur = ops[g & 1];
            Ops& nxt = ops[(g + 1) & 1];
            const unsigned char* addr[NL][4];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int b = 0; b < NL; ++b)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int m = (t * NL + b) * 2 + h;
                        acc[b][h] = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? cur.a1[t] : cur.a0[t], cur.b[b][t], acc[b][h], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (g + 1 < NGT) {
                            if (m == 0) {
#pragma unroll
                                for (int bq = 0; bq < NL; ++bq)
#pragma unroll
                                    for (int tq = 0; tq < 4; ++tq) addr[bq][tq] = bb[bq] + treg[g + 1][tq];
                                nxt.a0 = *reinterpret_cast<const floatx4*>(ap0 + 32 * (g + 1));
                                nxt.a1 = *reinterpret_cast<const floatx4*>(ap1 + 32 * (g + 1));
#pragma unroll
                                for (int bq = 0; bq < NL; ++bq)
#pragma unroll
                                    for (int tq = 0; tq < 4; ++tq) nxt.b[bq][tq] = *reinterpret_cast<const float*>(addr[bq][tq]);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
        }
    };

#pragma unroll 1
    for (int c = 0; c < P.chunks; ++c) {
        __syncthreads();                                // barrier c
        if (nlive > 0 && kp < P.NG) {                   // (a block past the tile multiplies cell 0)
            if constexpr (NGT > 0) multiply_unrolled(c & 1);
            else multiply(std::integral_constant<int, NBW>{}, c & 1);
        }
    }

    // ---- the parts of K meet in LDS (the stages are free: everybody has passed the last chunk)
    if constexpr (KS > 1) {
        __syncthreads();
        float* part = reinterpret_cast<float*>(smem);           // [K part - 1][block column][block][half][register][lane]
        if (kp > 0) {
#pragma unroll
            for (int b = 0; b < NBW; ++b)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        part[(((((kp - 1) * BW + wb) * NBW + b) * 2 + h) * 16 + v) * 64 + lane] = acc[b][h][v];
        }
        __syncthreads();
        if (kp > 0) return;
#pragma unroll
        for (int q = 0; q < KS - 1; ++q)
#pragma unroll
            for (int b = 0; b < NBW; ++b)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[b][h][v] += part[((((q * BW + wb) * NBW + b) * 2 + h) * 16 + v) * 64 + lane];
    }

    // ---- store: register v of a lane is output channel 8 (v / 4) + 4 kk + v % 4 of the 32-channel half, pixel lj
#pragma unroll
    for (int b = 0; b < NBW; ++b) {
        const int p = 32 * (BW * b + wb) + lj;
        if (b >= nlive || p >= valid_px) continue;
        const int i = fast_div(p, P.by_thwo), rem = p - i * thwo;
        const int ol = fast_div(rem, P.by_Wo), ow = rem - ol * P.Wo;
        float* yp = y + ((int64_t)(n0 + i) * P.C_out + co0) * HoWo + (row0 + ol) * P.Wo + ow;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int co = 32 * h + 8 * (v >> 2) + 4 * kk + (v & 3);
                if (co0 + co < P.C_out) yp[(int64_t)co * HoWo] = apply_epilogue(acc[b][h][v], co0 + co, P.ep);
            }
    }
}

struct DmaPlan {
    bool ok = false;
    int NBW = 0, BW = 4, KS = 1;
    size_t lds = 0;
    unsigned gx = 0, gy = 0;
    double est = 0;
    int64_t wgs = 0, work = 0;
    DmaParams P;
};

DmaPlan search_plan(const Conv2dShape& s, const void* x, const void* w)
{
    DmaPlan best;
    const int RS = s.R * s.S;
    const int64_t x_bytes = (int64_t)s.N * s.C_in * s.H * s.W * 4, w_bytes = (int64_t)s.C_out * s.C_in * RS * 4;
    if (s.C_in % 8 != 0 || x_bytes >= (1LL << 31) || w_bytes >= (1LL << 31)) return best;
    if (reinterpret_cast<uintptr_t>(w) % 16 != 0 || reinterpret_cast<uintptr_t>(x) % 4 != 0) return best;
    int CK0 = 8;
    while (CK0 * RS < 64 && CK0 < 32 && s.C_in % (2 * CK0) == 0) CK0 *= 2;
    const int co_blocks = (s.C_out + 63) / 64;
    if (co_blocks > 65535) return best;
    const int64_t IW = (int64_t)(s.Wo - 1) * s.stride + (int64_t)(s.S - 1) * s.dil + 1;
    const int HoWo = s.Ho * s.Wo;
    // a tile of NI whole images (tiles_y == 1) or of one of tiles_y equal runs of rows of one image (NI == 1)
    // BW block columns x KS parts of K (multiplying wavefronts), NBW blocks per wavefront
    auto consider = [&](int NBW, int BW, int KS, int NI, int tiles_y) {
        const int CK = CK0;
        const int PC = CK * RS / 4, PCp = PC | 1;
        if (PCp > 4 * kMaxFI || s.C_in % CK != 0 || CK * RS / 8 < KS) return;
        const int tp_max = 32 * BW * NBW;
        const int TH = (s.Ho + tiles_y - 1) / tiles_y;
        if ((int64_t)TH * s.Wo * NI > tp_max || (s.Ho + TH - 1) / TH != tiles_y) return;
        const int64_t IH = (int64_t)(TH - 1) * s.stride + (int64_t)(s.R - 1) * s.dil + 1;
        const int64_t WC = NI * IH * IW;
        if (WC > 64 * kMaxNS) return;
        const int NS = (int)((WC + 63) / 64);
        const size_t stage = (size_t)PCp * 1024 + (size_t)CK * NS * 256;
        const size_t lds = std::max(2 * stage + (size_t)CK * RS * 4, (size_t)(KS - 1) * BW * NBW * 8192);
        if (lds > kLdsBudget) return;
        const int blocks = (NI * TH * s.Wo + 31) / 32;
        const int64_t groups = (s.N + NI - 1) / NI;
        const int64_t wgs = groups * tiles_y * co_blocks;
        if (groups * tiles_y > 2147483647LL) return;
        if (KS > 1 && wgs > 256) return;                // (a K split holds its CU alone)
        // Periods (one block through all of K on one wavefront): those on a workgroup's critical path, and those of the
        // whole launch over the chip's 1024 SIMDs -- without a K split a workgroup holds BW SIMDs for its rounds whether
        // all of its wavefronts have a block or not, with one every wavefront works on every block.
        const int rounds = (blocks + BW - 1) / BW;
        const double est = KS == 1 ? std::max((double)rounds, (double)wgs * rounds * BW / 1024.0)
                                   : std::max((double)rounds / KS, (double)wgs * blocks / 1024.0);
        // equal estimates: the fewer block periods in all (blocks with dead lanes are wasted work), then as many CUs as
        // possible (every CU brings its own LDS and load path), then the fewer workgroups (filters are fetched per
        // workgroup), then the smaller split
        const int64_t work = wgs * blocks;
        if (best.ok) {
            const int64_t cus = std::min<int64_t>(wgs, 256), best_cus = std::min<int64_t>(best.wgs, 256);
            if (est > best.est) return;
            if (est == best.est) {
                if (work > best.work) return;
                if (work == best.work) {
                    if (cus < best_cus) return;
                    if (cus == best_cus && (wgs > best.wgs || (wgs == best.wgs && KS >= best.KS))) return;
                }
            }
        }
        best.work = work;
        best.ok = true;
        best.NBW = NBW;
        best.BW = BW;
        best.KS = KS;
        best.lds = lds;
        best.est = est;
        best.wgs = wgs;
        best.gx = (unsigned)(groups * tiles_y);
        best.gy = (unsigned)co_blocks;
        DmaParams& P = best.P;
        P.N = s.N; P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.Ho = s.Ho; P.Wo = s.Wo;
        P.stride = s.stride; P.pad = s.pad; P.dil = s.dil; P.S = s.S;
        P.CK = CK; P.RS = RS; P.NG = CK * RS / 8; P.PC = PC; P.PCp = PCp;
        P.NI = NI; P.TH = TH; P.tiles_y = tiles_y;
        P.IH = (int)IH; P.IW = (int)IW; P.cells_img = (int)(IH * IW);
        P.WC = (int)WC; P.NS = NS; P.WCp = 64 * NS;
        P.tile_px = NI * TH * s.Wo;
        P.chunks = s.C_in / CK;
        P.stage_bytes = (int)stage; P.win_off = PCp * 1024; P.tbl_off = (int)(2 * stage);
        P.x_bytes = (unsigned)x_bytes; P.w_bytes = (unsigned)w_bytes;
        P.by_tiles_y = make_fastdiv(tiles_y);
        P.by_cells_img = make_fastdiv(P.cells_img);
        P.by_IW = make_fastdiv(P.IW);
        P.by_thwo = make_fastdiv(TH * s.Wo);
        P.by_Wo = make_fastdiv(s.Wo);
        P.by_RS = make_fastdiv(RS);
        P.by_S = make_fastdiv(s.S);
        P.by_PCp = make_fastdiv(PCp);
    };
    if (IW > 64 * kMaxNS) return best;
    static const int kVariants[][3] = {{1, 4, 1}, {2, 4, 1}, {1, 4, 2}, {1, 2, 4}};      // NBW, BW, KS
    for (const auto& v : kVariants) {
        for (int NI = 2; NI <= s.N && (int64_t)NI * HoWo <= 32 * v[1] * v[0]; ++NI) consider(v[0], v[1], v[2], NI, 1);
        for (int tiles_y = 1; tiles_y <= s.Ho; ++tiles_y) consider(v[0], v[1], v[2], 1, tiles_y);
    }
    return best;
}

template <int NBW, int NGT, int BW, int KS>
hipError_t launch_dma(const float* x, const float* w, float* y, const DmaPlan& a, hipStream_t st)
{
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_dma_kernel<NBW, NGT, BW, KS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
    if (attr != hipSuccess) return attr;
    SW_NOTED_LAUNCH(note_kernel("mfma_f32_dma_kernel", 100 * KS + 10 * BW + NBW, a.P.CK, a.P.NI, a.P.TH),
                    (mfma_f32_dma_kernel<NBW, NGT, BW, KS>), dim3(a.gx, a.gy), dim3(64 * (BW * KS + 4)), a.lds, st, x, w, y, a.P);
    return hipGetLastError();
}

DmaPlan plan_dma(const Conv2dShape& s, const void* x, const void* w)
{
    thread_local PlanCache<DmaPlan> cache;
    return cache.get(s, PlanCache<DmaPlan>::low_bits(x, w, nullptr), [&] { return search_plan(s, x, w); });
}

}  // namespace

bool mfma_f32_dma_supported(const Conv2dShape& s, const float* x, const float* w) { return plan_dma(s, x, w).ok; }

hipError_t launch_mfma_f32_dma(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st, const Epilogue& ep)
{
    DmaPlan a = plan_dma(s, x, w);
    if (!a.ok) return hipErrorInvalidValue;
    a.P.ep = ep;
    if (a.KS == 4) return launch_dma<1, 0, 2, 4>(x, w, y, a, st);
    if (a.KS == 2) return launch_dma<1, 0, 4, 2>(x, w, y, a, st);
    if (a.NBW == 2) return launch_dma<2, 0, 4, 1>(x, w, y, a, st);
    if (a.P.NG == 9) return launch_dma<1, 9, 4, 1>(x, w, y, a, st);       // nine taps over chunks of eight channels
    return launch_dma<1, 0, 4, 1>(x, w, y, a, st);
}

}  // namespace swconv
