// Multi-channel fp32 convolution, stride 1, on the matrix cores.
//
// With more than one input channel every filter tap (r, s) is a small matrix, W_rs[co, ci], and the
// output tile is the sum over taps of W_rs times the input tile shifted by (r, s) (paper, section 3:
// sliding sums re-formulated as small matrix multiplications).  The shift is nothing but an address
// offset into the input tile staged in LDS, so no column matrix exists anywhere.
//
// Workgroup = 4 wavefronts = 64 output channels x one tile of TH x TW (<= 416) output pixels of one
// image, multiplied with v_mfma_f32_32x32x2_f32 (the form that sustains the fp32 matrix peak).
// Input channels are consumed in chunks of 16.  Per chunk the workgroup stages in LDS
//   the input window (tile + halo, zero-filled outside the image) as [ci/4][pixel][ci%4], and
//   the weights as [tap][ci/4][co][ci%4],
// so that one 16-byte LDS read hands a lane the operands of four matrix steps; the K index of those
// steps is permuted to match (step t of K-lane group g in octet o <-> channel 8o + 4g + t).
// The tile has 13 pixel blocks of 32.  Each wavefront owns one 32-channel block and six pixel
// blocks; the 13th block (the ragged tail) is split four ways, by channel block and by octet, and
// the two octet halves are added through LDS at the end, so every wavefront issues the same number
// of matrix instructions.  The next chunk is fetched from HBM/L2 into registers while the current one
// is multiplied, and the LDS operand reads of the next tap run ahead of the current tap's matrix
// instructions.
#include "swconv_internal.h"

namespace swconv {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kCK = 16;               // input channels per chunk
constexpr int kNFix = 6;              // whole pixel blocks per wavefront
constexpr int kSwing = 2 * kNFix;     // index of the shared 13th block
constexpr int kTilePx = (kSwing + 1) * 32;
constexpr int kLdsPx = 576;           // pixels of the staged input window (tile + halo)
constexpr int kXItems = 4 * kLdsPx / 256;
constexpr int kXBytes = 4 * kLdsPx * 16;
constexpr int kWGroupBytes = 64 * 16 + 64;   // one (tap, channel quad): 64 channels x 16 bytes, skewed

struct F32Params {
    Epilogue ep;                       // bias and rectifier of the EP variant
    int C_in, C_out, H, W, pad, Ho, Wo, TH, TW;
    FastDiv by_tiles_x, by_TW, by_IW, by_npx;
};

// DB: two LDS buffers, the next chunk is copied in while the current one is multiplied.
// EP: a per-channel bias and a rectifier are applied in the store (the plain variant carries no trace of them).
template <int R, int S, bool DB, bool EP>
__global__ __launch_bounds__(256, 1) void mfma_f32_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ w,
                                                          float* __restrict__ y, const F32Params P)
{
    constexpr int RS = R * S;
    constexpr int kBufBytes = kXBytes + RS * 4 * kWGroupBytes;      // one buffer: input window + weights
    constexpr int kSumOffset = (DB ? 2 : 1) * kBufBytes;            // 8 KB for the swing block's halves
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    floatx4* lx = reinterpret_cast<floatx4*>(smem);                 // [quad][pixel]
    unsigned char* lw = smem + kXBytes;                             // [tap][quad][co] floatx4, skewed

    const int C_in = P.C_in, C_out = P.C_out, H = P.H, W = P.W, pad = P.pad, Ho = P.Ho, Wo = P.Wo;
    const int TH = P.TH, TW = P.TW;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lg = lane >> 5, lj = lane & 31;       // K-lane group, row/column inside a 32 x 32 block
    // wave-uniform values are read into scalar registers so that tests on them are scalar branches
    const int wm = __builtin_amdgcn_readfirstlane(wave & 1);     // channel block
    const int wn = __builtin_amdgcn_readfirstlane(wave >> 1);    // pixel-block half and swing octet

    const int ty = fast_div(blockIdx.x, P.by_tiles_x);
    const int tx = blockIdx.x - ty * (int)P.by_tiles_x.d;
    // image index before channel block: workgroups that share an input tile get linear ids that are equal
    // modulo 8 when the tile count divides 8, i.e. they land on the same XCD and share its L2
    const int n = blockIdx.y;
    const int mb = blockIdx.z;

    const int row0 = ty * TH, col0 = tx * TW;
    const int IH = TH + R - 1, IW = TW + S - 1;
    const int npx = IH * IW;
    const int HW = H * W;
    const float* xn = x + (int64_t)n * C_in * HW;

    // ---- input staging plan: item = (channel quad q, window pixel) -----------------------------------
    int goff[kXItems];     // offset of channel 4q at that pixel inside one image; < 0: zero-fill
    int loff[kXItems];     // LDS slot; < 0: nothing to write
#pragma unroll
    for (int k = 0; k < kXItems; ++k) {
        const int idx = tid + 256 * k;
        const int q = fast_div(idx, P.by_npx);
        const int pix = idx - q * npx;
        const int e = fast_div(pix, P.by_IW), c = pix - e * IW;
        const int gr = row0 - pad + e, gc = col0 - pad + c;
        const bool live = idx < 4 * npx;
        const bool inside = live && gr >= 0 && gr < H && gc >= 0 && gc < W;
        goff[k] = inside ? (4 * q * H + gr) * W + gc : -1;
        loff[k] = live ? q * kLdsPx + pix : -1;
    }
    // ---- weight staging: thread = (output channel, channel quad): 4 x RS contiguous floats -----------
    const int sco = tid >> 2, sq = tid & 3;
    const float* wsrc = w + ((int64_t)((mb << 6) + sco) * C_in + 4 * sq) * RS;
    unsigned char* wdst = lw + sq * kWGroupBytes + sco * 16;

    // ---- operand addresses ---------------------------------------------------------------------------
    const int tile_px = TH * TW;
    int boff[kNFix + 1];       // LDS slot of this lane's pixel in quad lg, per pixel block (octet 0)
#pragma unroll
    for (int i = 0; i <= kNFix; ++i) {
        const int nb = i < kNFix ? wn * kNFix + i : kSwing;
        int p = nb * 32 + lj;
        if (p >= tile_px) p = 0;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        boff[i] = lg * kLdsPx + pi * IW + pj;
    }
    const unsigned char* aptr = lw + lg * kWGroupBytes + (32 * wm + lj) * 16;

    floatx16 acc[kNFix + 1];
#pragma unroll
    for (int i = 0; i <= kNFix; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    float xr[kXItems][4];
    floatx4 wr[RS];        // element t*RS + tap of the run <-> (channel t of the quad, tap)
    // A chunk travels global -> registers -> LDS in kXItems parts (one input item and a share of the weight
    // run each), so that the copies can be spread over the matrix instructions of the previous chunk.
    constexpr int WP = (RS + kXItems - 1) / kXItems;       // 16-byte weight groups per part
    auto fetch_part = [&](int c0, int part) {
        const float* xc = xn + (int64_t)c0 * HW;
#pragma unroll
        for (int t = 0; t < 4; ++t) {     // unconditional load at a clamped offset, then a select: no branch
            const float v = xc[max(goff[part], 0) + t * HW];
            xr[part][t] = goff[part] >= 0 ? v : 0.f;
        }
        const floatx4* ws = reinterpret_cast<const floatx4*>(wsrc + (int64_t)c0 * RS);
#pragma unroll
        for (int i = part * WP; i < (part + 1) * WP; ++i)
            if (i < RS) wr[i] = ws[i];
    };
    // registers -> LDS buffer `buf` (input window as it is, weights regrouped per tap: element t*RS + tap of
    // the run is channel t of the quad at that tap)
    auto stage_part = [&](int buf, int part) {
        if (loff[part] >= 0)
            lx[buf * (kBufBytes / 16) + loff[part]] = floatx4{xr[part][0], xr[part][1], xr[part][2], xr[part][3]};
#pragma unroll
        for (int tap = part * WP; tap < (part + 1) * WP; ++tap) {
            if (tap < RS)
                *reinterpret_cast<floatx4*>(wdst + buf * kBufBytes + tap * 4 * kWGroupBytes) =
                    floatx4{wr[tap / 4][tap % 4], wr[(RS + tap) / 4][(RS + tap) % 4],
                            wr[(2 * RS + tap) / 4][(2 * RS + tap) % 4], wr[(3 * RS + tap) / 4][(3 * RS + tap) % 4]};
        }
    };

    // operands of one (tap, octet) step from the LDS buffer at byte offset bofs: A for four K steps,
    // B for the six whole blocks and the swing block
    auto load_step = [&](int step, int bofs, floatx4& a, floatx4 (&b)[kNFix + 1]) {
        const int tap = step >> 1, o = step & 1;
        const int r = tap / S, q = tap - S * r;
        a = *reinterpret_cast<const floatx4*>(aptr + bofs + (tap * 4 + 2 * o) * kWGroupBytes);
        const int toff = (bofs >> 4) + 2 * o * kLdsPx + r * IW + q;
#pragma unroll
        for (int i = 0; i <= kNFix; ++i) b[i] = lx[boff[i] + toff];
    };
    // the same, one 16-byte read at a time: piece 0 is A, piece 1 + i is B of block i
    auto load_piece = [&](int step, int piece, int bofs, floatx4& a, floatx4 (&b)[kNFix + 1]) {
        const int tap = step >> 1, o = step & 1;
        const int r = tap / S, q = tap - S * r;
        if (piece == 0) a = *reinterpret_cast<const floatx4*>(aptr + bofs + (tap * 4 + 2 * o) * kWGroupBytes);
        else b[piece - 1] = lx[boff[piece - 1] + (bofs >> 4) + 2 * o * kLdsPx + r * IW + q];
    };
    auto load_swing = [&](int step, int bofs, floatx4& a, floatx4& b) {
        const int tap = step >> 1, o = step & 1;
        const int r = tap / S, q = tap - S * r;
        a = *reinterpret_cast<const floatx4*>(aptr + bofs + (tap * 4 + 2 * o) * kWGroupBytes);
        b = lx[boff[kNFix] + (bofs >> 4) + 2 * o * kLdsPx + r * IW + q];
    };
    auto load_pair = [&](int step, int pr, int bofs, floatx4& a, floatx4& b0, floatx4& b1) {
        const int tap = step >> 1, o = step & 1;
        const int r = tap / S, q = tap - S * r;
        a = *reinterpret_cast<const floatx4*>(aptr + bofs + (tap * 4 + 2 * o) * kWGroupBytes);
        const int toff = (bofs >> 4) + 2 * o * kLdsPx + r * IW + q;
        b0 = lx[boff[pr] + toff];
        b1 = lx[boff[pr + 1] + toff];
    };

    const int HoWo = Ho * Wo;
    float* yn = y + ((int64_t)n * C_out + (mb << 6) + 32 * wm + 4 * lg) * HoWo;
    float bv[16];                       // EP: the biases of this lane's 16 output channels (set before the stores)
    auto store_block = [&](int nb, const floatx16& c) {
        const int p = nb * 32 + lj;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        const int oi = row0 + pi, oj = col0 + pj;
        if (p < tile_px && oi < Ho && oj < Wo) {
            float* dst = yn + oi * Wo + oj;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float t = c[v];
                if (EP) {
                    t += bv[v];
                    if (P.ep.relu) t = fmaxf(t, 0.0f);
                }
                dst[(8 * (v >> 2) + (v & 3)) * HoWo] = t;
            }
        }
    };

    constexpr int NSTEP = 2 * RS;
    // steps FETCH_AT .. +kXItems-1 issue the next chunk's global loads, one part each; with two LDS buffers
    // steps STAGE_AT .. +kXItems-1 copy them into the other buffer
    constexpr int FETCH_AT = 0;
    constexpr int STAGE_AT = NSTEP - kXItems;
    static_assert(STAGE_AT >= FETCH_AT + kXItems || !DB, "a part must be fetched before it is staged");
    const int chunks = C_in / kCK;
#pragma unroll
    for (int part = 0; part < kXItems; ++part) fetch_part(0, part);
#pragma unroll
    for (int part = 0; part < kXItems; ++part) stage_part(0, part);
    __syncthreads();
    for (int ch = 0; ch + 1 < chunks; ++ch) {
        const int buf = DB ? (ch & 1) : 0;
        const int bofs = buf * kBufBytes;
        floatx4 a[2];
        floatx4 b[2][kNFix + 1];
        load_step(0, bofs, a[0], b[0]);
#pragma unroll
        for (int step = 0; step < NSTEP; ++step) {
            const int cur = step & 1;
            // Everything that is not a matrix instruction -- the LDS reads of the next step's operands, one part
            // of the next chunk's global loads, one part of its copy into the other LDS buffer -- is issued one
            // instruction group at a time between the matrix instructions, whose pipe runs on meanwhile.
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int i = 0; i < kNFix; ++i) {
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b[cur][i][t], acc[i], 0, 0, 0);
                    const int slot = t * kNFix + i;
                    if (step + 1 < NSTEP && slot <= kNFix + 1) load_piece(step + 1, slot, bofs, a[cur ^ 1], b[cur ^ 1]);
                    if (slot == kNFix + 2 && step >= FETCH_AT && step < FETCH_AT + kXItems)
                        fetch_part((ch + 1) * kCK, step - FETCH_AT);
                    if (slot == kNFix + 6 && DB && step >= STAGE_AT) stage_part(buf ^ 1, step - STAGE_AT);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if ((step & 1) == wn)               // the swing block: only this wavefront's octet
                    acc[kNFix] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b[cur][kNFix][t], acc[kNFix], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
        if (!DB) {
#pragma unroll
            for (int part = 0; part < kXItems; ++part) stage_part(0, part);
            __syncthreads();
        }
    }

    // ---- last chunk: block by block, so that finished blocks are stored while the next ones multiply ----
    if (EP) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
            bv[v] = P.ep.bias ? P.ep.bias[(mb << 6) + 32 * wm + 4 * lg + 8 * (v >> 2) + (v & 3)] : 0.0f;
    }
    {
        const int bofs = (DB ? ((chunks - 1) & 1) : 0) * kBufBytes;
        // swing block first: this wavefront's octet, then the two octet halves meet in LDS
        {
            floatx4 a[2], bs[2];
            load_swing(wn, bofs, a[0], bs[0]);
#pragma unroll
            for (int tap = 0; tap < RS; ++tap) {
                const int cur = tap & 1;
                if (tap + 1 < RS) load_swing(2 * (tap + 1) + wn, bofs, a[cur ^ 1], bs[cur ^ 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[kNFix] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], bs[cur][t], acc[kNFix], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float* lsum = reinterpret_cast<float*>(smem + kSumOffset);
        if (wn == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) lsum[(wm * 16 + v) * 64 + lane] = acc[kNFix][v];
        }
        __syncthreads();
        if (wn == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[kNFix][v] += lsum[(wm * 16 + v) * 64 + lane];
            store_block(kSwing, acc[kNFix]);
        }
        // whole blocks in pairs: two independent accumulators alternate
#pragma unroll
        for (int pr = 0; pr < kNFix; pr += 2) {
            floatx4 a[2], b0[2], b1[2];
            load_pair(0, pr, bofs, a[0], b0[0], b1[0]);
#pragma unroll
            for (int step = 0; step < NSTEP; ++step) {
                const int cur = step & 1;
                if (step + 1 < NSTEP) load_pair(step + 1, pr, bofs, a[cur ^ 1], b0[cur ^ 1], b1[cur ^ 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    acc[pr] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b0[cur][t], acc[pr], 0, 0, 0);
                    acc[pr + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b1[cur][t], acc[pr + 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            store_block(wn * kNFix + pr, acc[pr]);
            store_block(wn * kNFix + pr + 1, acc[pr + 1]);
        }
    }
}

struct Tiling {
    int TH, TW, tiles_x, tiles_y;
};

Tiling pick_tiling(const Conv2dShape& s)
{
    Tiling t;
    const int splits = (s.Wo + 63) / 64;
    t.TW = (s.Wo + splits - 1) / splits;
    t.TH = kTilePx / t.TW;
    if (t.TH > s.Ho) t.TH = s.Ho;
    while (t.TH > 1 && (t.TH + s.R - 1) * (t.TW + s.S - 1) > kLdsPx) --t.TH;
    const int bands = (s.Ho + t.TH - 1) / t.TH;
    t.TH = (s.Ho + bands - 1) / bands;      // equal row bands
    t.tiles_x = (s.Wo + t.TW - 1) / t.TW;
    t.tiles_y = (s.Ho + t.TH - 1) / t.TH;
    return t;
}

constexpr int kLdsMax = 160 * 1024;
constexpr int kSumBytes = 2 * 16 * 64 * 4;
constexpr int buf_bytes(int RS) { return kXBytes + RS * 4 * kWGroupBytes; }

template <int R, int S, bool EP>
hipError_t launch(const float* x, const float* w, float* y, const Conv2dShape& s, const Tiling& t, hipStream_t st,
                  const Epilogue& ep)
{
    constexpr bool DB = 2 * buf_bytes(R * S) + kSumBytes <= kLdsMax;
    constexpr int bytes = (DB ? 2 : 1) * buf_bytes(R * S) + kSumBytes;
    static_assert(bytes <= kLdsMax, "LDS budget");
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_kernel<R, S, DB, EP>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (attr != hipSuccess) return attr;
    F32Params P;
    P.ep = ep;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = t.TH; P.TW = t.TW;
    P.by_tiles_x = make_fastdiv(t.tiles_x);
    P.by_TW = make_fastdiv(t.TW);
    P.by_IW = make_fastdiv(t.TW + S - 1);
    P.by_npx = make_fastdiv((t.TH + R - 1) * (t.TW + S - 1));
    dim3 grid((unsigned)(t.tiles_x * t.tiles_y), (unsigned)s.N, (unsigned)(s.C_out / 64));
    SW_NOTED_LAUNCH(note_kernel("mfma_f32_kernel", (int)(R), (int)(S), (int)(DB), (int)(EP)), (mfma_f32_kernel<R, S, DB, EP>), grid, dim3(256), bytes, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_supported(const Conv2dShape& s)
{
    if (s.stride != 1 || s.dil != 1 || s.C_in % kCK != 0 || s.C_out % 64 != 0) return false;
    if (!((s.R == 3 && s.S == 3) || (s.R == 5 && s.S == 5))) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    const Tiling t = pick_tiling(s);
    if ((t.TH + s.R - 1) * (t.TW + s.S - 1) > kLdsPx || t.TH * t.TW > kTilePx) return false;
    return (int64_t)t.tiles_x * t.tiles_y <= 65535 && s.C_out / 64 <= 65535 && s.N <= 65535;
}

int64_t mfma_f32_workgroups(const Conv2dShape& s)
{
    const Tiling t = pick_tiling(s);
    if (t.TH * t.TW < kTilePx / 2) return 0;       // images so small that a tile stays half empty
    return (int64_t)t.tiles_x * t.tiles_y * s.N * (s.C_out / 64);
}

hipError_t launch_mfma_f32(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st,
                           const Epilogue& ep)
{
    if (reinterpret_cast<uintptr_t>(w) % 16 != 0) return launch_direct_conv2d_f32(x, w, y, s, false, st, &ep);
    const Tiling t = pick_tiling(s);
    if (ep.bias || ep.relu) {
        if (s.R == 3) return launch<3, 3, true>(x, w, y, s, t, st, ep);
        return launch<5, 5, true>(x, w, y, s, t, st, ep);
    }
    if (s.R == 3) return launch<3, 3, false>(x, w, y, s, t, st, ep);
    return launch<5, 5, false>(x, w, y, s, t, st, ep);
}

}  // namespace swconv
