// Convolution layer of a Hadamard-binarised network (HadaNets section 3.2: activations binarised along
// the width with beta_a, filters along their flattened C*KH*KW with beta_w) on the matrix cores, with
// filters prepared ahead of time and the activation fragments read straight from a patch in LDS.
//
//   out[b, n, oz, oy] = sum_{c, dz, dy} A~[b, c, oz*stride - pad + dz, oy*stride - pad + dy] * W~[n, c, dz, dy]
//
// with A~ = scale * sign of the activation (0 outside the input) and W~ = scale * sign of the filter
// weight.  Both are fp32 numbers.  Two forms of the product (FORM):
//   0  each number is split exactly into three bf16 pieces and the six largest of the nine piece products are
//      added on v_mfma_f32_32x32x16_bf16 (what is dropped is below 2^-24 of a term);
//   1  each number is scaled by a power of two into the range of fp16 and split into two fp16 pieces, h =
//      the number rounded, m = the remainder rounded (22 significant bits together), and hm, mh, hh are added
//      on v_mfma_f32_32x32x16_f16: half the multiplies, |error| <= 3 * 2^-22 of a term (plus 2^-39 of the
//      largest activation / weight met so far, where a remainder falls below fp16's smallest subnormal).  The
//      power of two is per filter for the weights (fixed at preparation) and per workgroup for the
//      activations: the exponent of the largest magnitude among the channel groups staged so far; when a
//      later group raises it the accumulators are rescaled (exactly) before that group is multiplied.
// Because both sides are plain numbers here, the sum over k may run in any order, and the order chosen
// is (channel group of 32, filter tap, channel inside the group).  One K stage is then one tap of one
// channel group: 32 channels at a fixed offset (dz, dy) from every output position.
//
// Filters.  They do not change between calls, so their pieces are produced once by
// conv_prepare_filters_kernel, in the order in which a wave consumes them: for a block of 32 filters, a
// channel group, a tap, an MFMA step of 16 channels and a piece, 64 x 16 bytes = the B operand of one
// MFMA (lane l: filter l mod 32, channels 8 (l div 32) .. + 7).  In the layer kernel a wave loads these
// operands straight from memory into registers, two stages ahead, with 1 KB contiguous per instruction;
// filters never pass through LDS and cost no arithmetic per workgroup.  They are the MFMA's first operand
// and the activations its second: a lane's 16 results are then 16 filters at one position and a half wave
// holds 32 consecutive positions, which is how the B x N x OH x OW output is laid out -- it is stored
// straight from the accumulators.
//
// Activations.  A workgroup owns R whole output rows of one image (R * OW <= 128 positions) and a tile
// of 64 or 128 filters.  For the current channel group it keeps the input patch those rows need --
// ((R - 1) stride + KH) rows x ((OW - 1) stride + KW) columns, zero outside the image -- in LDS as
// three planes of bf16 pieces (two of fp16 in FORM 1), 32 channels contiguous per pixel (pixel stride 80
// bytes: the 16-byte fragment reads of neighbouring positions fall on distinct banks).  The A operand of position m,
// tap (dz, dy), channels 8j .. 8j+7 is one 16-byte LDS read at
//     pixel(m) + dz * PW + dy,   pixel(m) = (orow * stride) * PW + oy * stride,
// so every activation is fetched, rebuilt and split once per workgroup and channel group and read KH*KW
// times by the multiply itself: no operand tile is assembled, and the only barrier is the one per
// channel group that hands over the next patch (fetched after the first tap of a group, written after
// its last one -- into the other buffer when two fit, else between two barriers; FORM 1 has one more per
// group, for the exchange of the largest magnitude).  For 3 x 3 windows the nine taps of a group are
// written out and the next patch is split and written item by item between the multiplies of the last
// taps, so that the vector instructions are issued while the matrix pipe works.
#include <type_traits>

#include "bf16_pieces.h"
#include "kernels.h"
#include "wave_ops.h"

namespace hbmm {
namespace {

constexpr int kGroup = 32;                  // channels per group = K elements per stage
constexpr int kPixBytes = 80;               // 32 bf16 + 16 bytes of padding
constexpr int kNumXcdD = 8;
constexpr int kThreadsD = 512;
constexpr int kPatchArea = 160 * 1024 - 512;   // LDS of a workgroup, all of it patch (and, after the multiply, the exchange of the two halves of K)
constexpr int kOperandBytes = 1024;         // one MFMA B operand: 64 lanes x 16 bytes
// filters of one stage for one block of 32: 2 steps x 3 (bf16) or 2 (fp16) pieces
constexpr int stage_bytes(int form) { return 2 * (form == 0 ? 3 : 2) * kOperandBytes; }
constexpr int kTargetExp = 14;              // FORM 1: the largest magnitude is scaled into [2^14, 2^15)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// FORM 1 helpers.  e is the biased exponent of the largest magnitude, kept in [14, 254] so that the
// multiplier 2^(14 - (e - 127)) is a normal float (anything smaller than 2^-113 is treated as 0).
__device__ __forceinline__ int norm_exponent(uint32_t max_abs_bits)
{
    const int e = (int)(max_abs_bits >> 23);
    return e < 14 ? 14 : (e > 254 ? 254 : e);
}
__device__ __forceinline__ float norm_factor(int e) { return __builtin_bit_cast(float, (uint32_t)(268 - e) << 23); }
// v (already scaled) as two fp16 patterns in the low halves of hi and mid.
__device__ __forceinline__ void split2_f16(float v, uint32_t &hi, uint32_t &mid)
{
    const _Float16 h = (_Float16)v;
    const _Float16 m = (_Float16)(v - (float)h);
    hi = __builtin_bit_cast(uint16_t, h);
    mid = __builtin_bit_cast(uint16_t, m);
}
// The three piece pairs (x piece, y piece) of FORM 1, smallest contributions first.
constexpr int kPiecePairs2[3][2] = {{0, 1}, {1, 0}, {0, 0}};
constexpr int kMaxItems = 5;                // staging items per thread (a stride-2 3 x 3 layer on 56 x 56 needs 513 pixels = 5)

// ------------------------------------------------------------------------------------------------
// Filter preparation: one thread per (block of 32 filters, group, tap, step, lane) writes the three
// pieces of its 8 values.  Filters past N and channels past C are written as zeros.
struct PrepareArgs {
    const uint32_t *w_bits;      // unused with beta = 1
    const float *w_scales;       // beta = 1: the filters themselves, N x K
    unsigned char *pieces;
    int64_t ldw, lds;
    int32_t N, C, KK;
    int32_t groups;
    uint32_t magic;              // ceil(2^32 / beta): k div beta = umulhi(k, magic) for k < 2^24
    int32_t raw;                 // beta = 1
    int64_t total;               // threads that have work
    int32_t *exps;               // FORM 1: biased exponent per filter (32 * blocks entries), inside `pieces`
    int32_t nscales;             // FORM 1: entries of a row of w_scales that belong to the filter
};

// FORM 1, first step: one wave per filter finds the exponent of its largest magnitude (of its scales, or of
// its weights when unquantised).  Filters past N get the smallest exponent (their pieces are zeros).
__global__ __launch_bounds__(64) void conv_filter_exponents_kernel(const PrepareArgs a)
{
    const int n = blockIdx.x, lane = threadIdx.x;
    uint32_t mx = 0;
    if (n < a.N)
        for (int i = lane; i < a.nscales; i += 64)
            mx = max(mx, __builtin_bit_cast(uint32_t, a.w_scales[(int64_t)n * a.lds + i]) & 0x7fffffffu);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, d));
    if (lane == 0) a.exps[n] = norm_exponent(mx);
}

template <int FORM>
__global__ __launch_bounds__(256) void conv_prepare_filters_kernel(const PrepareArgs a)
{
    constexpr int NP = FORM == 0 ? 3 : 2;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= a.total) return;
    const int lane = (int)(id & 63);
    int64_t r = id >> 6;
    const int ks = (int)(r & 1);
    r >>= 1;
    const int t = (int)(r % a.KK);
    r /= a.KK;
    const int g = (int)(r % a.groups);
    const int cb = (int)(r / a.groups);
    const int n = cb * 32 + (lane & 31);
    const int c0 = g * kGroup + ks * 16 + (lane >> 5) * 8;
    const int64_t nrow = n < a.N ? n : a.N - 1;
    uint32_t h[8], m[8], l[8];
    float norm = 1.f;
    if constexpr (FORM == 1) norm = norm_factor(a.exps[n]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = c0 + i;
        const bool live = n < a.N && c < a.C;
        const uint32_t k = (uint32_t)(live ? c * a.KK + t : 0);
        float v;
        if (a.raw) {
            v = a.w_scales[nrow * a.lds + k];
        } else {
            const float s = a.w_scales[nrow * a.lds + __umulhi(k, a.magic)];
            const uint32_t word = a.w_bits[nrow * a.ldw + (k >> 5)];
            v = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, s) ^ (~(word >> (k & 31)) << 31));
        }
        if constexpr (FORM == 0) {
            split3(live ? v : 0.f, h[i], m[i], l[i]);
        } else {
            split2_f16(live ? v * norm : 0.f, h[i], m[i]);
            l[i] = 0;
        }
    }
    u32x4 dh, dm, dl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if constexpr (FORM == 0) {
            dh[i] = pair16(h[2 * i], h[2 * i + 1]);
            dm[i] = pair16(m[2 * i], m[2 * i + 1]);
            dl[i] = pair16(l[2 * i], l[2 * i + 1]);
        } else {
            dh[i] = h[2 * i] | (h[2 * i + 1] << 16);
            dm[i] = m[2 * i] | (m[2 * i + 1] << 16);
        }
    }
    unsigned char *dst = a.pieces + ((((int64_t)cb * a.groups + g) * a.KK + t) * 2 + ks) * (NP * kOperandBytes) + lane * 16;
    *reinterpret_cast<u32x4 *>(dst) = dh;
    *reinterpret_cast<u32x4 *>(dst + kOperandBytes) = dm;
    if constexpr (FORM == 0) *reinterpret_cast<u32x4 *>(dst + 2 * kOperandBytes) = dl;
}

// ------------------------------------------------------------------------------------------------
// x div d for the small non-negative x of the kernel's set-up (x * d < 2^32): m = ceil(2^32 / d), or 0 for d = 1.
__device__ __forceinline__ int small_div(int x, uint32_t m) { return m ? (int)__umulhi((uint32_t)x, m) : x; }

struct ConvDirectArgs {
    const uint32_t *x_bits;
    const float *x_scales;
    const unsigned char *pieces;
    const int32_t *exps;         // FORM 1: biased exponent per filter
    float *out;
    int32_t Y, yblocks;          // filters, and blocks of 32 of them in `pieces`
    int32_t beta_x, nseg, HS;    // activation segment length, segments per row ceil(W / beta_x), H * nseg
    int32_t C, H, W, HW, OH, OW, OHW, KW, KK, stride, pad;
    int32_t CHW, CHS;            // elements and scales of one image: C * H * W, C * H * nseg
    int64_t bits_bytes, scales_bytes;   // bytes of the activation words and scales: what the buffer loads may touch
    int32_t R, tiles_per_image, tiles_y, tiles_total, slots_per_xcd;
    int32_t B, G;                // images, and images per tile (1 unless a whole image is at most 64 positions)
    int32_t PI, IP;              // patch pixels and tile positions of one image: P = G * PI, positions = G * IP
    int32_t PW, P;               // patch width and pixels
    uint32_t m_P, m_PI, m_PW, m_IP, m_OW, m_beta;   // divisors of the set-up as multipliers, see small_div()
    int32_t plane;               // bytes of one piece plane of the patch: P * 80
    int32_t patch_bufs;          // 2: group g lives in buffer g & 1; 1: one buffer, refilled between two barriers
    int32_t groups;              // ceil(C / 32)
    uint32_t sign;               // 0x80000000; 0 when the tensor is unquantised (then x_scales holds the values)
};

// XI: pixels a lane stages per channel group (for one octet of channels); XI * 128 >= P.
// Eight waves on a tile of 128 positions; every wave owns 64 positions x 32 filters.
// NTY = 2 (128 filters): 2 x 4 wave tiles, each wave takes both MFMA steps of a stage;
// NTY = 1 (64 filters): 2 x 2 wave tiles, waves 0-3 take the first step of every stage and waves 4-7 the
//      second; the two halves are added through LDS at the end.
template <int XI, int NTY, int FORM>
__global__ __launch_bounds__(kThreadsD) void conv_direct_kernel(const ConvDirectArgs a)
{
    constexpr int NP = FORM == 0 ? 3 : 2;            // pieces per number
    constexpr int NQ = FORM == 0 ? 6 : 3;            // piece products per MFMA step
    constexpr int kStageBytes = stage_bytes(FORM);
    constexpr int NT = 64 * NTY;
    constexpr int TX = 2;
    constexpr int WV = kThreadsD / 64;
    constexpr int KS = NTY == 1 ? 1 : 2;     // MFMA steps a wave takes per stage
    constexpr int kWavesY = NTY == 1 ? 2 : 4;   // waves side by side along the filters
    __shared__ __attribute__((aligned(16))) unsigned char sPatch[kPatchArea];
    __shared__ uint32_t sMax[WV];                     // FORM 1: largest magnitude staged by each wave

    const int slot_id = (blockIdx.x % kNumXcdD) * a.slots_per_xcd + blockIdx.x / kNumXcdD;
    if (slot_id >= a.tiles_total) return;
    const int tile_x = slot_id / a.tiles_y, y0 = (slot_id % a.tiles_y) * NT;
    // (with several images per tile every image is whole: tiles_per_image = 1, oz0 = 0)
    const int img = (tile_x / a.tiles_per_image) * a.G, oz0 = (tile_x % a.tiles_per_image) * a.R;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // wave -> (filter block, position half, MFMA step): the fastest index runs along the filters
    const int wcol0 = (wave % kWavesY) * 32;
    const int wrow0 = ((wave / kWavesY) & 1) * 64;
    const int ks0 = NTY == 1 ? wave / (WV / 2) : 0;       // first MFMA step of a stage this wave takes
    const int npos = a.G * a.IP;                            // positions of a full tile (<= 128)

    // ---- role 1: patch staging.  A wave stages one octet of channels (wave mod 4) for half of the patch's pixels:
    // item j of a lane is pixel (wave div 4) * 64 + lane + 128 j.  The channel of an element is then the same for
    // the whole wave, so everything that depends on it is scalar arithmetic, and the loads are buffer loads --
    // descriptor + 32-bit lane offset (+ a scalar offset for the channel) -- whose range check returns 0 for a
    // pixel outside the image: such a pixel is given an offset past the end of the buffer and costs no test.
    const int oct = wave & 3;
    const int64_t e_base = (int64_t)img * a.CHW;          // first element of the tile's first image
    const int64_t w_base = e_base >> 5;                   // ... the word that holds its bit
    const int64_t s_base = (int64_t)img * a.CHS;          // ... its first scale
    auto records = [](int64_t bytes) { return (int)(uint32_t)(bytes < 0 ? 0 : bytes > 0xffffff00ll ? 0xffffff00ll : bytes); };
    const __amdgpu_buffer_rsrc_t rsrc_bits = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t *>(a.x_bits) + w_base, 0, records(a.bits_bytes - 4 * w_base), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_scales = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.x_scales) + s_base, 0, records(a.scales_bytes - 4 * s_base), 0x00020000);
    constexpr uint32_t kPastEnd = 0xfffffffcu;            // a byte offset no buffer reaches
    uint32_t perel[XI];  // element index of channel 0 at the item's pixel, counted from the bit of the tile's first element
    uint32_t poob[XI];   // 0, or kPastEnd for a pixel outside the image (or-ed into the word's byte offset)
    uint32_t psoff[XI];  // byte offset of channel 0's scale at the item's pixel (kPastEnd outside the image)
    int pdst[XI];        // byte offset of the item inside a plane; -1: the item does not exist
#pragma unroll
    for (int j = 0; j < XI; ++j) {
        const int pix = (wave >> 2) * 64 + lane + j * 128;
        const int pc = min(pix, a.P - 1);
        const int gi = small_div(pc, a.m_PI), lp = pc - gi * a.PI;   // image of the tile, pixel inside its patch
        const int prow = small_div(lp, a.m_PW), pcol = lp - prow * a.PW;
        const int z = oz0 * a.stride - a.pad + prow, y = pcol - a.pad;
        const bool inside = pix < a.P && img + gi < a.B && z >= 0 && z < a.H && y >= 0 && y < a.W;
        const int row = gi * a.C * a.H + z;               // row of channel 0, counted from the tile's first image
        pdst[j] = pix < a.P ? pix * kPixBytes + oct * 16 : -1;
        poob[j] = inside ? 0u : kPastEnd;
        perel[j] = inside ? (uint32_t)(row * a.W + y) + (uint32_t)(e_base & 31) : 0u;
        // segments run along the width of a row and start anew in every row (the last one may be shorter)
        psoff[j] = inside ? (uint32_t)(row * a.nseg + small_div(y, a.m_beta)) * 4u : kPastEnd;
    }
    struct PatchRegs {
        uint32_t w[XI][8];
        float s[XI][8];
    };
    // channel c = 32 g + 8 oct + i of item j: element perel + c * HW, scale psoff + 4 c * HS
    auto fetch_patch = [&](PatchRegs &r, int g) __attribute__((always_inline)) {
        const int c0 = g * kGroup + oct * 8;
        auto one = [&](int j, int i) __attribute__((always_inline)) {
            const uint32_t e = perel[j] + (uint32_t)((c0 + i) * a.HW);
            r.w[j][i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rsrc_bits, (int)((((e >> 5) << 2)) | poob[j]), 0, 0);
            r.s[j][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc_scales, (int)psoff[j], (c0 + i) * a.HS * 4, 0));
        };
        if (c0 + 8 <= a.C) {
#pragma unroll
            for (int j = 0; j < XI; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) one(j, i);
        } else {
            // the last group of a channel count that is not a multiple of 8: channels past C are zeros
#pragma unroll
            for (int j = 0; j < XI; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    r.w[j][i] = 0u;
                    r.s[j][i] = 0.f;
                    if (c0 + i < a.C) one(j, i);
                }
        }
    };
    // FORM 1: the largest magnitude among the values this thread holds (what was not loaded is 0)
    auto patch_max = [&](const PatchRegs &r) __attribute__((always_inline)) {
        uint32_t mx = 0;
#pragma unroll
        for (int j = 0; j < XI; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) mx = max(mx, __builtin_bit_cast(uint32_t, r.s[j][i]) & 0x7fffffffu);
        return mx;
    };
    // One element (channel i of item j) of group g as pieces; then the item's eight elements written to the planes.
    auto park_elem = [&](const PatchRegs &r, int j, int i, int g, float norm, uint32_t (&h)[8], uint32_t (&m)[8], uint32_t (&l)[8])
                         __attribute__((always_inline)) {
        // value = scale with the sign of the element's bit (1: positive); the bit sits at position e mod 32
        // of the word, and a shift by (not e) mod 32 = 31 - e mod 32 brings its complement to the sign
        const uint32_t e = perel[j] + (uint32_t)((g * kGroup + oct * 8 + i) * a.HW);
        const uint32_t minus = (~r.w[j][i] << (~e & 31u)) & a.sign;
        const uint32_t value = __builtin_bit_cast(uint32_t, r.s[j][i]) ^ minus;
        if constexpr (FORM == 0) {
            split3(__builtin_bit_cast(float, value), h[i], m[i], l[i]);
        } else {
            split2_f16(__builtin_bit_cast(float, value) * norm, h[i], m[i]);
            l[i] = 0;
        }
    };
    auto park_write = [&](int j, unsigned char *buf, const uint32_t (&h)[8], const uint32_t (&m)[8], const uint32_t (&l)[8])
                          __attribute__((always_inline)) {
        if (pdst[j] >= 0) {
            u32x4 dh, dm, dl;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (FORM == 0) {
                    dh[i] = pair16(h[2 * i], h[2 * i + 1]);
                    dm[i] = pair16(m[2 * i], m[2 * i + 1]);
                    dl[i] = pair16(l[2 * i], l[2 * i + 1]);
                } else {
                    dh[i] = h[2 * i] | (h[2 * i + 1] << 16);
                    dm[i] = m[2 * i] | (m[2 * i + 1] << 16);
                }
            }
            unsigned char *dst = buf + pdst[j];
            *reinterpret_cast<u32x4 *>(dst) = dh;
            *reinterpret_cast<u32x4 *>(dst + a.plane) = dm;
            if constexpr (FORM == 0) *reinterpret_cast<u32x4 *>(dst + 2 * a.plane) = dl;
        }
    };
    auto park_item = [&](const PatchRegs &r, int j, int g, unsigned char *buf, float norm) __attribute__((always_inline)) {
        uint32_t h[8], m[8], l[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) park_elem(r, j, i, g, norm, h, m, l);
        park_write(j, buf, h, m, l);
    };
    auto park_patch = [&](const PatchRegs &r, int g, unsigned char *buf, float norm) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < XI; ++j) park_item(r, j, g, buf, norm);
    };

    // ---- role 2: multiply.  Lane l feeds position row (l mod 32) and channels 8 (l div 32) .. + 7 of a step.
    int xoff[TX];   // byte offset of the lane's position (window corner) and channel octet inside a plane
#pragma unroll
    for (int tx = 0; tx < TX; ++tx) {
        const int ml = min(wrow0 + tx * 32 + (lane & 31), npos - 1);
        const int gi = small_div(ml, a.m_IP), lm = ml - gi * a.IP;
        const int orow = small_div(lm, a.m_OW), oy = lm - orow * a.OW;
        xoff[tx] = (gi * a.PI + (orow * a.stride) * a.PW + oy * a.stride) * kPixBytes + (lane >> 5) * 16 + ks0 * 32;
    }
    // filter operands of this wave's block of 32 filters: stage s at s * kStageBytes (a block past the last
    // one re-reads the last: its columns are never stored)
    const unsigned char *ysrc = a.pieces + (int64_t)min((y0 + wcol0) >> 5, a.yblocks - 1) * a.groups * a.KK * kStageBytes +
                                ks0 * (NP * kOperandBytes) + lane * 16;
    const int nstages = a.groups * a.KK;
    struct FilterRegs {
        u32x4 f[KS][NP];
    };
    auto fetch_filter = [&](FilterRegs &r, int stage) __attribute__((always_inline)) {
        const unsigned char *src = ysrc + (int64_t)min(stage, nstages - 1) * kStageBytes;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int p = 0; p < NP; ++p)
                r.f[ks][p] = *reinterpret_cast<const u32x4 *>(src + (ks * NP + p) * kOperandBytes);
    };

    f32x16 res[TX];
#pragma unroll
    for (int tx = 0; tx < TX; ++tx)
#pragma unroll
        for (int v = 0; v < 16; ++v) res[tx][v] = 0.f;

    const int patch_stride = a.patch_bufs == 2 ? NP * a.plane : 0;
    PatchRegs xr;
    FilterRegs ya, yb, yc;
    // FORM 1: e_run is the exponent that the patches staged so far are scaled by (it only grows)
    int e_run = 14;
    float norm = 1.f;
    // Every wave publishes the largest magnitude it holds of group g; after a barrier all of them agree
    // on the exponent.  If it grew, what has been accumulated so far is rescaled to the new unit.
    auto publish_max = [&](int g) __attribute__((always_inline)) {
        uint32_t mx = patch_max(xr);
        mx = max(mx, dpp_u32<kDppQuadSwap1>(mx));
        mx = max(mx, dpp_u32<kDppQuadSwap2>(mx));
        mx = max(mx, dpp_u32<kDppHalfMirror>(mx));
        mx = max(mx, dpp_u32<kDppRowMirror>(mx));
        mx = max(mx, (uint32_t)__shfl_xor((int)mx, 16));
        mx = max(mx, (uint32_t)__shfl_xor((int)mx, 32));
        if (lane == 0) sMax[wave] = mx;
    };
    auto agreed_exponent = [&]() __attribute__((always_inline)) {
        uint32_t all = 0;
#pragma unroll
        for (int w = 0; w < WV; ++w) all = max(all, sMax[w]);
        return max(e_run, norm_exponent(__builtin_amdgcn_readfirstlane(all)));
    };
    auto adopt_exponent = [&](int e_new) __attribute__((always_inline)) {
        if (e_new != e_run) {
#pragma unroll
            for (int tx = 0; tx < TX; ++tx)
#pragma unroll
                for (int v = 0; v < 16; ++v) res[tx][v] = __builtin_amdgcn_ldexpf(res[tx][v], e_run - e_new);
            e_run = e_new;
        }
        norm = norm_factor(e_run);
    };
    auto agree_on_exponent = [&]() __attribute__((always_inline)) { adopt_exponent(agreed_exponent()); };
    fetch_patch(xr, 0);
    fetch_filter(ya, 0);
    fetch_filter(yb, 1);
    // FORM 1: lane l keeps the exponent of filter (l mod 32) of this wave's block for the store (requested here,
    // where its latency costs nothing)
    int filter_exp = 0;
    if constexpr (FORM == 1) filter_exp = a.exps[min(y0 + wcol0 + (lane & 31), a.yblocks * 32 - 1)];
    if constexpr (FORM == 1) {
        publish_max(0);
        __syncthreads();
        agree_on_exponent();
    }
    park_patch(xr, 0, sPatch, norm);
    __syncthreads();

    // ---- 3 x 3 windows with room for two patches: the nine taps of a channel group written out, so that the staging
    // of the next group -- the exchange of the maxima (FORM 1) and the splitting of one item per tap -- sits in the
    // same straight-line code as a tap's multiplies and its vector instructions are issued between them (in the
    // general loop below it runs after the group's last multiply, with the matrix pipe idle).  Not with four or
    // five items per lane: holding them across the written-out taps spills registers (measured: slower).
    constexpr bool kUnrolled3x3 = XI <= 3;
    bool unrolled = false;
    if constexpr (kUnrolled3x3) unrolled = a.KK == 9 && a.KW == 3 && a.patch_bufs == 2;
    if constexpr (kUnrolled3x3) if (unrolled) {
        // `item` >= 0: this tap also splits item `item` of the next group's patch, one element after every eighth of
        // its multiplies (fenced, so that the order holds): the element's vector instructions are issued while
        // the matrix pipe works on the MFMAs before them.  `extra` runs after the multiplies.
        auto tap = [&](const FilterRegs &cur, FilterRegs &next, int g_, int k, int stage_, auto item_c, unsigned char *nbuf,
                       float item_norm, auto &&extra) __attribute__((always_inline)) {
            constexpr int item = decltype(item_c)::value;
            constexpr int NM = KS * NQ * TX;
            fetch_filter(next, stage_ + 2);
            __builtin_amdgcn_sched_barrier(0);
            const unsigned char *px = sPatch + (g_ & 1) * patch_stride + ((k / 3) * a.PW + k % 3) * kPixBytes;
            u32x4 fx[KS][NP][TX];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int p = 0; p < NP; ++p)
#pragma unroll
                    for (int tx = 0; tx < TX; ++tx)
                        fx[ks][p][tx] = *reinterpret_cast<const u32x4 *>(px + p * a.plane + xoff[tx] + ks * 32);
            uint32_t h[8], m[8], l[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
#pragma unroll
                for (int idx = c * NM / 8; idx < (c + 1) * NM / 8; ++idx) {
                    const int ks = idx / (NQ * TX), q = (idx / TX) % NQ, tx = idx % TX;
                    if constexpr (FORM == 0)
                        res[tx] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, cur.f[ks][kPiecePairs[q][1]]),
                            __builtin_bit_cast(bf16x8, fx[ks][kPiecePairs[q][0]][tx]), res[tx], 0, 0, 0);
                    else
                        res[tx] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(f16x8, cur.f[ks][kPiecePairs2[q][1]]),
                            __builtin_bit_cast(f16x8, fx[ks][kPiecePairs2[q][0]][tx]), res[tx], 0, 0, 0);
                }
                if constexpr (item >= 0) {
                    park_elem(xr, item, c, g_ + 1, item_norm, h, m, l);
                    // (pinned: without a use here the optimiser sinks the arithmetic to the write after the last MFMA)
                    if constexpr (FORM == 0)
                        asm volatile("" : "+v"(h[c]), "+v"(m[c]), "+v"(l[c]));
                    else
                        asm volatile("" : "+v"(h[c]), "+v"(m[c]));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (item >= 0) park_write(item, nbuf, h, m, l);
            extra();
        };
        // taps 9 - XI .. 8 each split one item of the next patch; FORM 1 publishes its maxima with tap 7 - XI and
        // agrees on the exponent (one barrier) before tap 9 - XI
        constexpr int kFirstPark = 9 - XI;
        int e_next = e_run;
        float norm_next = norm;
        auto group = [&](auto more_c, int g_) __attribute__((always_inline)) {
            constexpr bool more = decltype(more_c)::value;
            const int s0 = g_ * 9;
            unsigned char *nbuf = sPatch + ((g_ + 1) & 1) * patch_stride;
            auto staged = [&](auto k_c) __attribute__((always_inline)) {
                constexpr int k = decltype(k_c)::value;
                if constexpr (more) {
                    if constexpr (FORM == 1 && k == kFirstPark - 2) publish_max(g_ + 1);
                }
            };
#define HBMM_TAP(K, CUR, NEXT)                                                              \
    do {                                                                                    \
        if constexpr (more && FORM == 1 && K == kFirstPark) {                               \
            __syncthreads();                                                                \
            e_next = agreed_exponent();                                                     \
            norm_next = norm_factor(e_next);                                                \
        }                                                                                   \
        tap(CUR, NEXT, g_, K, s0 + K, std::integral_constant<int, (more && K >= kFirstPark) ? K - kFirstPark : -1>{}, nbuf, \
            norm_next, [&]() __attribute__((always_inline)) { staged(std::integral_constant<int, K>{}); });               \
        if constexpr (more && K == 0) fetch_patch(xr, g_ + 1);                              \
    } while (0)
            HBMM_TAP(0, ya, yc);
            HBMM_TAP(1, yb, ya);
            HBMM_TAP(2, yc, yb);
            HBMM_TAP(3, ya, yc);
            HBMM_TAP(4, yb, ya);
            HBMM_TAP(5, yc, yb);
            HBMM_TAP(6, ya, yc);
            HBMM_TAP(7, yb, ya);
            HBMM_TAP(8, yc, yb);
#undef HBMM_TAP
            if constexpr (more) {
                __syncthreads();   // the next patch is complete, and every wave has read the last tap of this one
                if constexpr (FORM == 1) adopt_exponent(e_next);
            }
        };
        for (int g_ = 0; g_ + 1 < a.groups; ++g_) group(std::true_type{}, g_);
        group(std::false_type{}, a.groups - 1);
    }

    int g = 0, t = 0, dz = 0, dy = 0, stage = 0;
    if (unrolled) stage = a.groups * a.KK;   // done above
    // One stage: request the filter operands of the stage after next into `next`, multiply with `cur`.
    // (Two stages ahead: a stage of a 64-filter tile is only 12 MFMAs per wave, shorter than a trip to L2.)
    auto run_stage = [&](const FilterRegs &cur, FilterRegs &next) __attribute__((always_inline)) {
        const bool more = g + 1 < a.groups;
        fetch_filter(next, stage + 2);
        // (without this fence the scheduler sinks the loads below the multiplies to save registers, and the
        // next stage then waits out their whole latency)
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char *px = sPatch + (g & 1) * patch_stride + (dz * a.PW + dy) * kPixBytes;
        // (FORM 1: the next group's largest magnitude is published before the last tap's multiplies, so that the
        // exchange is over when the barrier after them is reached; a single tap has no earlier place)
        if constexpr (FORM == 1)
            if (more && a.KK > 1 && t == a.KK - 1) publish_max(g + 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 fx[NP][TX];
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int tx = 0; tx < TX; ++tx)
                    fx[p][tx] = *reinterpret_cast<const u32x4 *>(px + p * a.plane + xoff[tx] + ks * 32);
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int tx = 0; tx < TX; ++tx) {
                    // (filters as the first operand: a lane's 16 results are then 16 filters at one position, and
                    // the lanes of a half wave run along positions, which is how the output is laid out)
                    if constexpr (FORM == 0)
                        res[tx] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, cur.f[ks][kPiecePairs[q][1]]),
                            __builtin_bit_cast(bf16x8, fx[kPiecePairs[q][0]][tx]), res[tx], 0, 0, 0);
                    else
                        res[tx] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(f16x8, cur.f[ks][kPiecePairs2[q][1]]),
                            __builtin_bit_cast(f16x8, fx[kPiecePairs2[q][0]][tx]), res[tx], 0, 0, 0);
                }
        }
        // the next group's activations: requested once the first tap's multiplies are queued, so that the
        // loads are the youngest in flight and nothing before the last tap waits for them
        if (t == 0 && more) fetch_patch(xr, g + 1);
        ++stage;
        if (++dy == a.KW) {
            dy = 0;
            ++dz;
        }
        if (++t == a.KK) {
            if (more) {
                if constexpr (FORM == 1) {
                    if (a.KK == 1) publish_max(g + 1);
                    __syncthreads();   // (also the barrier that a single patch buffer needs here)
                    agree_on_exponent();
                } else if (a.patch_bufs == 1) {
                    __syncthreads();   // every wave has read the last tap of this group
                }
                park_patch(xr, g + 1, sPatch + ((g + 1) & 1) * patch_stride, norm);
                __syncthreads();
            }
            t = dz = dy = 0;
            ++g;
        }
    };
    while (stage < nstages) {
        run_stage(ya, yc);
        if (stage < nstages) run_stage(yb, ya);
        if (stage < nstages) run_stage(yc, yb);
    }

    // ---- store: out is B x Y x OH x OW.  Lane l of an accumulator tile holds position (l mod 32) and the 16 filters
    // 8 (v div 4) + 4 (l div 32) + (v mod 4): for each v a half wave writes 32 consecutive positions of one filter.
    if (NTY == 1) {
        // add the two halves of K: the second half of the waves hands its accumulators to the first through the
        // patch area (every wave must have left the multiply loop before it is reused)
        __syncthreads();
        float *half = reinterpret_cast<float *>(sPatch) + (wave % (WV / 2)) * (TX * 16 * 64);
        if (wave >= WV / 2) {
#pragma unroll
            for (int tx = 0; tx < TX; ++tx)
#pragma unroll
                for (int v = 0; v < 16; ++v) half[(tx * 16 + v) * 64 + lane] = res[tx][v];
        }
        __syncthreads();
        if (wave >= WV / 2) return;
#pragma unroll
        for (int tx = 0; tx < TX; ++tx)
#pragma unroll
            for (int v = 0; v < 16; ++v) res[tx][v] += half[(tx * 16 + v) * 64 + lane];
    }
    // FORM 1: back to the caller's units: 2^(e_run - 127 - 14) for the activations times the filter's own
    int unscale[16];
    if constexpr (FORM == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int f = 8 * (v >> 2) + (v & 3);
            const int e0 = __builtin_amdgcn_readlane(filter_exp, f), e1 = __builtin_amdgcn_readlane(filter_exp, f + 4);
            unscale[v] = (lane < 32 ? e0 : e1) + e_run - 2 * (127 + kTargetExp);
        }
    }
#pragma unroll
    for (int tx = 0; tx < TX; ++tx) {
        const int ml = wrow0 + tx * 32 + (lane & 31);
        const int mc = min(ml, npos - 1);
        const int gi = small_div(mc, a.m_IP), lm = mc - gi * a.IP;
        const int orow = small_div(lm, a.m_OW), oy = lm - orow * a.OW;
        const bool pos_ok = ml < npos && img + gi < a.B && oz0 + orow < a.OH;
        float *dst = a.out + ((int64_t)(img + gi) * a.Y * a.OH + (oz0 + orow)) * a.OW + oy;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int col = y0 + wcol0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            float val = res[tx][v];
            if constexpr (FORM == 1) val = __builtin_amdgcn_ldexpf(val, unscale[v]);
            if (pos_ok && col < a.Y) dst[(int64_t)col * a.OHW] = val;
        }
    }
}

// Rows of output per workgroup: as many as fill 128 positions, fewer if the patch would not fit the LDS or
// would take more than 5 staging items per thread; 0 if not even one row fits.
int rows_per_tile(const ConvGeometry &g, int64_t OH, int64_t OW, int form)
{
    const int np = form == 0 ? 3 : 2;
    if (OW > 128) return 0;
    const int PW = (int)(OW - 1) * g.stride + g.KW;
    int R = (int)(128 / OW < OH ? 128 / OW : OH);
    auto pixels = [&](int r) { return ((r - 1) * g.stride + g.KH) * PW; };
    while (R >= 1 && (4 * pixels(R) > kMaxItems * kThreadsD || np * pixels(R) * kPixBytes > kPatchArea)) --R;
    return R;
}

}  // namespace

// Bytes of the pieces proper; FORM 1 appends one exponent (int32) per filter of the 32-filter blocks.
static int64_t pieces_proper_bytes(int64_t N, int64_t C, int KH, int KW, int form)
{
    return ((N + 31) / 32) * ((C + kGroup - 1) / kGroup) * KH * KW * (int64_t)stage_bytes(form);
}

int64_t conv_filter_pieces_bytes(int64_t N, int64_t C, int KH, int KW, int form)
{
    return pieces_proper_bytes(N, C, KH, KW, form) + (form == 0 ? 0 : ((N + 31) / 32) * 32 * (int64_t)sizeof(int32_t));
}

hipError_t launch_conv_prepare_filters(const uint32_t *w_bits, const float *w_scales, int64_t ldw, int64_t lds, int beta,
                                       int64_t N, int64_t C, int KH, int KW, int form, void *pieces, hipStream_t s)
{
    PrepareArgs a{};
    a.w_bits = w_bits; a.w_scales = w_scales; a.pieces = static_cast<unsigned char *>(pieces);
    a.ldw = ldw; a.lds = lds;
    a.N = (int32_t)N; a.C = (int32_t)C; a.KK = KH * KW;
    a.groups = (int32_t)((C + kGroup - 1) / kGroup);
    a.raw = beta == 1 ? 1 : 0;
    a.magic = beta == 1 ? 0u : (uint32_t)(((1ull << 32) + beta - 1) / beta);
    a.total = ((N + 31) / 32) * a.groups * a.KK * 2 * 64;
    const int64_t blocks = (a.total + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (form == 0) {
        conv_prepare_filters_kernel<0><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
        return hipGetLastError();
    }
    a.exps = reinterpret_cast<int32_t *>(a.pieces + pieces_proper_bytes(N, C, KH, KW, form));
    const int64_t K = C * KH * KW;
    a.nscales = (int32_t)(beta == 1 ? K : (K + beta - 1) / beta);
    conv_filter_exponents_kernel<<<dim3((unsigned)((N + 31) / 32 * 32)), dim3(64), 0, s>>>(a);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    conv_prepare_filters_kernel<1><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

bool conv_direct_fits(const ConvGeometry &g)
{
    const int64_t OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1, OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
    return rows_per_tile(g, OH, OW, 0) >= 1;   // (the two-piece form needs less room)
}

hipError_t launch_conv_direct(const ConvActivations &x, const void *pieces, int64_t N, const ConvGeometry &g, int form,
                              float *out, hipStream_t s)
{
    const int np = form == 0 ? 3 : 2;
    const int64_t OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1, OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
    const int KK = g.KH * g.KW;
    const int PW = (int)(OW - 1) * g.stride + g.KW;
    int R = rows_per_tile(g, OH, OW, form);
    if (R < 1) return hipErrorNotSupported;
    const int tiles_per_image = (int)((OH + R - 1) / R);
    R = (int)((OH + tiles_per_image - 1) / tiles_per_image);   // even rows per tile
    const int threads = kThreadsD;
    const int PI = ((R - 1) * g.stride + g.KH) * PW;
    // small feature maps (a whole image is at most 64 positions: the 7 x 7 maps of a network's last stage): several
    // images per tile, each with its own patch, so that the 128 position rows of the tile are not mostly empty
    int G = 1;
    if (tiles_per_image == 1)
        while ((G + 1) * R * OW <= 128 && G + 1 <= g.B && 4 * (G + 1) * PI <= kMaxItems * kThreadsD &&
               2 * np * (G + 1) * PI * kPixBytes <= kPatchArea)
            ++G;
    const int P = G * PI;
    const int bufs = 2 * np * P * kPixBytes <= kPatchArea ? 2 : 1;
    const int64_t tiles_x = (g.B + G - 1) / G * tiles_per_image;
    // filters per tile: 128, or 64 when there are no more or when 128 would leave compute units without a workgroup
    const int nty = N <= 64 || tiles_x * ((N + 127) / 128) < 256 ? 1 : 2;
    const int64_t tiles_y = (N + 64 * nty - 1) / (64 * nty);
    const int64_t total = tiles_x * tiles_y, per_xcd = (total + kNumXcdD - 1) / kNumXcdD;
    if (per_xcd * kNumXcdD > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    ConvDirectArgs a{};
    // beta = 1: `scales` is the unquantised tensor.  It then plays both parts: read as the "scale" of
    // element e (segment length 1) it is the value itself, sign included, and the sign taken from the
    // bit word is switched off; the word loads still happen and are pointed at the same memory.
    a.x_bits = x.beta == 1 ? reinterpret_cast<const uint32_t *>(x.scales) : x.bits;
    a.x_scales = x.scales; a.sign = x.beta == 1 ? 0u : 0x80000000u;
    a.beta_x = x.beta; a.nseg = (int32_t)((g.W + x.beta - 1) / x.beta); a.HS = (int32_t)(g.H * a.nseg);
    // (the buffer loads address the images of one tile with 32-bit byte offsets)
    if ((double)G * (double)g.C * (double)g.H * (double)g.W * 4.0 > 4.0e9) return hipErrorNotSupported;
    a.CHW = (int32_t)(g.C * g.H * g.W); a.CHS = (int32_t)(g.C * a.HS);
    a.bits_bytes = (g.B * g.C * g.H * g.W + 31) / 32 * 4;
    a.scales_bytes = g.B * g.C * (int64_t)a.HS * 4;
    a.pieces = static_cast<const unsigned char *>(pieces);
    a.exps = reinterpret_cast<const int32_t *>(a.pieces + pieces_proper_bytes(N, g.C, g.KH, g.KW, form));
    a.out = out; a.Y = (int32_t)N; a.yblocks = (int32_t)((N + 31) / 32);
    a.C = (int32_t)g.C; a.H = (int32_t)g.H; a.W = (int32_t)g.W; a.HW = (int32_t)(g.H * g.W);
    a.OH = (int32_t)OH; a.OW = (int32_t)OW; a.OHW = (int32_t)(OH * OW);
    a.KW = g.KW; a.KK = KK; a.stride = g.stride; a.pad = g.pad;
    a.R = R; a.tiles_per_image = tiles_per_image; a.tiles_y = (int32_t)tiles_y; a.tiles_total = (int32_t)total;
    a.slots_per_xcd = (int32_t)per_xcd;
    a.B = (int32_t)g.B; a.G = G; a.PI = PI; a.IP = (int32_t)(R * OW);
    a.PW = PW; a.P = P; a.plane = P * kPixBytes; a.patch_bufs = bufs;
    auto magic = [](int d) { return d == 1 ? 0u : (uint32_t)(((1ull << 32) + d - 1) / d); };   // 0 stands for d = 1
    a.m_P = magic(P); a.m_PI = magic(PI); a.m_PW = magic(PW); a.m_IP = magic(a.IP); a.m_OW = magic((int)OW);
    a.m_beta = magic(x.beta);
    a.groups = (int32_t)((g.C + kGroup - 1) / kGroup);
    const int xi = (P + 127) / 128;
    const dim3 grid((unsigned)(per_xcd * kNumXcdD)), block(threads);
#define HBMM_DIRECT_LAUNCH(I)                                           \
    do {                                                                \
        if (form == 0) {                                                \
            if (nty == 1)                                               \
                conv_direct_kernel<I, 1, 0><<<grid, block, 0, s>>>(a);  \
            else                                                        \
                conv_direct_kernel<I, 2, 0><<<grid, block, 0, s>>>(a);  \
        } else {                                                        \
            if (nty == 1)                                               \
                conv_direct_kernel<I, 1, 1><<<grid, block, 0, s>>>(a);  \
            else                                                        \
                conv_direct_kernel<I, 2, 1><<<grid, block, 0, s>>>(a);  \
        }                                                               \
    } while (0)
    if (xi <= 1)
        HBMM_DIRECT_LAUNCH(1);
    else if (xi == 2)
        HBMM_DIRECT_LAUNCH(2);
    else if (xi == 3)
        HBMM_DIRECT_LAUNCH(3);
    else if (xi == 4)
        HBMM_DIRECT_LAUNCH(4);
    else
        HBMM_DIRECT_LAUNCH(5);
#undef HBMM_DIRECT_LAUNCH
    return hipGetLastError();
}

}  // namespace hbmm
