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
    int C_in, C_out, H, W, pad, Ho, Wo, TH, TW;
    FastDiv by_tiles_x, by_TW, by_IW, by_npx;
};

template <int R, int S>
__global__ __launch_bounds__(256, 1) void mfma_f32_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ w,
                                                          float* __restrict__ y, const F32Params P)
{
    constexpr int RS = R * S;
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
    auto fetch = [&](int c0) {
        const float* xc = xn + (int64_t)c0 * HW;
#pragma unroll
        for (int k = 0; k < kXItems; ++k) {
#pragma unroll
            for (int t = 0; t < 4; ++t) xr[k][t] = goff[k] >= 0 ? xc[goff[k] + t * HW] : 0.f;
        }
        const floatx4* ws = reinterpret_cast<const floatx4*>(wsrc + (int64_t)c0 * RS);
#pragma unroll
        for (int i = 0; i < RS; ++i) wr[i] = ws[i];
    };

    // operands of one (tap, octet) step: A for four K steps, B for the six whole blocks and the swing block
    auto load_step = [&](int step, floatx4& a, floatx4 (&b)[kNFix + 1]) {
        const int tap = step >> 1, o = step & 1;
        const int r = tap / S, q = tap - S * r;
        a = *reinterpret_cast<const floatx4*>(aptr + (tap * 4 + 2 * o) * kWGroupBytes);
        const int toff = 2 * o * kLdsPx + r * IW + q;
#pragma unroll
        for (int i = 0; i <= kNFix; ++i) b[i] = lx[boff[i] + toff];
    };

    fetch(0);
    const int chunks = C_in / kCK;
    for (int ch = 0; ch < chunks; ++ch) {
#pragma unroll
        for (int k = 0; k < kXItems; ++k)
            if (loff[k] >= 0) lx[loff[k]] = floatx4{xr[k][0], xr[k][1], xr[k][2], xr[k][3]};
        {
            float f[4 * RS];
#pragma unroll
            for (int i = 0; i < RS; ++i) {
                f[4 * i + 0] = wr[i].x; f[4 * i + 1] = wr[i].y; f[4 * i + 2] = wr[i].z; f[4 * i + 3] = wr[i].w;
            }
#pragma unroll
            for (int tap = 0; tap < RS; ++tap)
                *reinterpret_cast<floatx4*>(wdst + tap * 4 * kWGroupBytes) =
                    floatx4{f[tap], f[RS + tap], f[2 * RS + tap], f[3 * RS + tap]};
        }
        __syncthreads();
        if (ch + 1 < chunks) fetch((ch + 1) * kCK);

        floatx4 a[2];
        floatx4 b[2][kNFix + 1];
        load_step(0, a[0], b[0]);
#pragma unroll
        for (int step = 0; step < 2 * RS; ++step) {
            const int cur = step & 1;
            if (step + 1 < 2 * RS) load_step(step + 1, a[cur ^ 1], b[cur ^ 1]);
            __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the matrix instructions
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int i = 0; i < kNFix; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b[cur][i][t], acc[i], 0, 0, 0);
                if ((step & 1) == wn)               // the swing block: only this wavefront's octet
                    acc[kNFix] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][t], b[cur][kNFix][t], acc[kNFix], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
    }

    // ---- the two octet halves of the swing block meet in LDS -------------------------------------------
    float* lsum = reinterpret_cast<float*>(smem);
    if (wn == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) lsum[(wm * 16 + v) * 64 + lane] = acc[kNFix][v];
    }
    __syncthreads();
    if (wn == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[kNFix][v] += lsum[(wm * 16 + v) * 64 + lane];
    }

    // ---- store: register v of a lane is channel 8*(v/4) + 4*lg + v%4 of the block, pixel lj ---------------
    const int HoWo = Ho * Wo;
    float* yn = y + ((int64_t)n * C_out + (mb << 6) + 32 * wm + 4 * lg) * HoWo;
#pragma unroll
    for (int i = 0; i <= kNFix; ++i) {
        if (i == kNFix && wn != 0) break;
        const int nb = i < kNFix ? wn * kNFix + i : kSwing;
        const int p = nb * 32 + lj;
        const int pi = fast_div(p, P.by_TW), pj = p - pi * TW;
        const int oi = row0 + pi, oj = col0 + pj;
        if (p < tile_px && oi < Ho && oj < Wo) {
            float* dst = yn + oi * Wo + oj;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                dst[(8 * (v >> 2) + (v & 3)) * HoWo] = acc[i][v];
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

int lds_bytes(int RS) { return kXBytes + RS * 4 * kWGroupBytes; }

template <int R, int S>
hipError_t launch(const float* x, const float* w, float* y, const Conv2dShape& s, const Tiling& t, hipStream_t st)
{
    const int bytes = lds_bytes(R * S);
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_f32_kernel<R, S>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (attr != hipSuccess) return attr;
    F32Params P;
    P.C_in = s.C_in; P.C_out = s.C_out; P.H = s.H; P.W = s.W; P.pad = s.pad; P.Ho = s.Ho; P.Wo = s.Wo;
    P.TH = t.TH; P.TW = t.TW;
    P.by_tiles_x = make_fastdiv(t.tiles_x);
    P.by_TW = make_fastdiv(t.TW);
    P.by_IW = make_fastdiv(t.TW + S - 1);
    P.by_npx = make_fastdiv((t.TH + R - 1) * (t.TW + S - 1));
    dim3 grid((unsigned)(t.tiles_x * t.tiles_y), (unsigned)s.N, (unsigned)(s.C_out / 64));
    hipLaunchKernelGGL((mfma_f32_kernel<R, S>), grid, dim3(256), bytes, st, x, w, y, P);
    return hipGetLastError();
}

}  // namespace

bool mfma_f32_supported(const Conv2dShape& s)
{
    if (s.stride != 1 || s.C_in % kCK != 0 || s.C_out % 64 != 0) return false;
    if (!((s.R == 3 && s.S == 3) || (s.R == 5 && s.S == 5))) return false;
    if ((int64_t)s.C_in * s.H * s.W > 2147483647LL) return false;
    const Tiling t = pick_tiling(s);
    if ((t.TH + s.R - 1) * (t.TW + s.S - 1) > kLdsPx || t.TH * t.TW > kTilePx) return false;
    return (int64_t)t.tiles_x * t.tiles_y <= 65535 && s.C_out / 64 <= 65535 && s.N <= 65535;
}

hipError_t launch_mfma_f32(const float* x, const float* w, float* y, const Conv2dShape& s, hipStream_t st)
{
    if (reinterpret_cast<uintptr_t>(w) % 16 != 0) return launch_direct_conv2d_f32(x, w, y, s, false, st);
    const Tiling t = pick_tiling(s);
    if (s.R == 3) return launch<3, 3>(x, w, y, s, t, st);
    return launch<5, 5>(x, w, y, s, t, st);
}

}  // namespace swconv
