// HBMM on the matrix cores for the cases where one operand is not reduced to bits per 32-bit
// word: beta_a = 1 (the paper's HBWN: activations stay fp32) and short segments (beta < 32, the
// settings HadaNets trains with: 2, 4, 8, 16).
//
//   out[x, y] = sum_j sY[y, j] * sum_{k in segment j of Y} X~[x, k] * (+-1)_Y[y, k]
//
// X is the "dense" side: X~[x, k] is an fp32 number, either the raw operand (beta_x = 1) or
// sX[x, k div beta_x] * Sign(x) rebuilt from the packed bits and scales (Eq. 2 / Eq. 4 of the
// paper).  Y is the "sign" side: +-1 per element, its scale applied once per segment (beta_y >= 16).
// With short segments the popcount formulation costs five vector-ALU instructions per segment per
// output; here the cost does not depend on beta_x at all.
//
// The inner sum is a dense contraction, so it runs on v_mfma_f32_32x32x16_bf16.  An fp32 value is
// split exactly into three bf16 pieces (8 + 8 + 8 significant bits: hi = top half of the fp32
// pattern, mid = top half of (v - hi), lo = v - hi - mid); +-1 is exact in bf16; so every product is
// exact and the three piece-products accumulate in the MFMA's fp32 accumulator: a segment sum is an
// fp32 sum of exact terms, like the scalar definition.  At the end of a Y segment one FMA per
// output applies sY and the next segment's first MFMA starts from a zero accumulator.
//
// Layout of the work.  Workgroup = 8 waves, tile 128 (X) x 256 (Y); wave = 64 x 64 = 2 x 2 MFMA tiles
// (lane l feeds row (l mod 32) and 8 consecutive k at 8 * (l div 32); both operands use the same
// map).  K is walked in stages of 32:
//   * X: raw mode fetches 128 rows x 32 fp32 with 16-byte loads; packed mode fetches one word of bits
//     and the 1..4 scales that cover a thread's 8 elements.  Either way the three bf16 pieces are
//     produced once per workgroup while the stage is parked in LDS (row stride 80 bytes: the 16-byte
//     fragment reads of 8 consecutive rows land on distinct banks).  In packed mode only the scale is
//     split; the sign is a xor on the piece's sign bit.
//   * Y: one packed word per row per stage; two threads expand it to 32 bf16 values +-1.0 in LDS
//     (three ALU instructions per pair of elements), shared by the waves that use that row.
// Global loads are unconditional (indices clamped, never guarded, so the compiler knows how many
// are outstanding) and run three stages ahead through three rotating register sets: a stage is
// only ~16 KB per workgroup and HBM latency is several stages long.  Tiles that share X rows get
// consecutive slots on one XCD so that the repeat reads of X come from that XCD's L2.
#include "bf16_pieces.h"
#include "kernels.h"

namespace hbmm {
namespace {

constexpr int kBX = 128, kBY = 256;
constexpr int kThreadsS = 512;
constexpr int kStageK = 32;
constexpr int kRowBytes = 80;                     // 32 bf16 + 16 bytes of padding
constexpr int kPieceBytes = kBX * kRowBytes;      // one bf16 piece of the X tile
constexpr int kNumXcdS = 8;

// X modes: how the dense side is given
constexpr int kXRaw = 0;      // fp32 operand itself (beta_x = 1)
constexpr int kXScale1 = 1;   // packed, beta_x >= 8: one scale covers a thread's 8 elements
constexpr int kXScale2 = 2;   // packed, beta_x = 4: two scales per 8 elements
constexpr int kXScale4 = 3;   // packed, beta_x = 2: four scales per 8 elements
constexpr int kXConv = 4;     // packed activation tensor read through a convolution window (see below)
constexpr int kXAny = 5;      // any beta_x (1 included), any K: a scale looked up per element (see kYAny)

// Sign masks for `n` (<= 8) pairs of elements: complemented bit 2i of `inv` -> bit 15 of dword i,
// complemented bit 2i+1 -> bit 31 (the sign positions of a pair of bf16 values).
template <int PAIRS>
__device__ __forceinline__ void sign_masks(uint32_t inv, uint32_t (&m)[PAIRS])
{
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) m[i] = ((inv << (15 - 2 * i)) | (inv << (30 - 2 * i))) & 0x80008000u;
}

// The three bf16 piece rows of 8 consecutive elements of a packed operand: `byte` holds their sign
// bits (1 = +), `sc` the SPT scales that cover them (8 / SPT elements each).  Only the scales are
// split; the sign is a xor on each piece's sign bit.
template <int SPT>
__device__ __forceinline__ void packed_pieces(uint32_t byte, const float (&sc)[SPT], u32x4 &dh, u32x4 &dm, u32x4 &dl)
{
    uint32_t sm[4];
    sign_masks<4>(~byte & 0xffu, sm);
    uint32_t ph[SPT], pm[SPT], pl[SPT];
#pragma unroll
    for (int j = 0; j < SPT; ++j) {
        uint32_t h, m, l;
        split3(sc[j], h, m, l);
        ph[j] = pair16(h, h);
        pm[j] = pair16(m, m);
        pl[j] = pair16(l, l);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = i * SPT / 4;    // scale that covers elements 2i, 2i+1
        dh[i] = ph[j] ^ sm[i];
        dm[i] = pm[j] ^ sm[i];
        dl[i] = pl[j] ^ sm[i];
    }
}

struct SplitArgs {
    const float *x_raw;          // kXRaw
    const uint32_t *x_bits;      // packed modes
    const float *x_scales;
    const uint32_t *y_bits;
    const float *y_scales;
    float *out;
    int64_t ldx_raw, ld_out_x, ld_out_y;
    int32_t ldw_x, lds_x, ldw_y, lds_y;
    int32_t X, Y, K;
    int32_t log2_beta_x;         // packed modes
    int32_t log2_beta_y;         // Y as pieces
    int32_t stages_per_yseg;     // beta_y / 32 (beta_y >= 32); unused when beta_y = 16
    int32_t log2_stages_per_yseg;
    int32_t tiles_y, tiles_total, slots_per_xcd;
    // kXConv: X row m = (b * OH + oz) * OW + oy is an output position, k = (c * KH + dz) * KW + dy a
    // filter tap; X~[m, k] is the binarised activation at (b, c, oz*stride - pad + dz,
    // oy*stride - pad + dy), or 0 outside the input.  x_bits / x_scales hold the whole tensor packed
    // flat (element e: bit e mod 32 of word e div 32, scale e div beta_a; beta_a divides W, so a
    // segment never leaves its row).  The output is B x Y x OH x OW.
    int32_t cv_c, cv_h, cv_w, cv_hw, cv_ow, cv_ohw, cv_kw, cv_kk, cv_stride, cv_pad;
    int32_t cv_magic_kk, cv_magic_kw;   // 65536 / d + 1: (t * magic) >> 16 == t / d for t < 64, d <= 32
    int32_t cv_q32, cv_r32;             // 32 div KK, 32 mod KK: how (c, tap) moves from stage to stage
    uint32_t cv_sign;                   // 0x80000000; 0 when the tensor is unquantised (see launch_mfma_split_conv)
    // kXAny / kYAny
    uint32_t any_magic_x, any_magic_y;  // ceil(2^32 / beta)
    uint32_t any_sign_x;                // 0x80000000; 0 when X is the raw operand
    int32_t any_x_raw;                  // X is raw: x_scales is the operand itself, x_bits is never used
};

// Y modes: how the other side is given
constexpr int kYSign = 0;     // packed, beta_y >= 32: +-1 per element, its scale applied once per segment
constexpr int kYSign16 = 1;   // packed, beta_y = 16: the same with a segment per MFMA step
constexpr int kYPieces1 = 2;  // packed, beta_y = 8: a segment is shorter than an MFMA step, so Y is rebuilt as fp32
constexpr int kYPieces2 = 3;  // packed, beta_y = 4   values and split into pieces like X; the six largest of the
constexpr int kYPieces4 = 4;  // packed, beta_y = 2   nine piece products are added and there is no epilogue
// Segment lengths that are not powers of two, and K that is not a multiple of 32 or of beta: both sides
// are rebuilt as fp32 values element by element (scale index k div beta by a multiply-high with
// ceil(2^32 / beta), exact for k < 2^24), elements at k >= K are parked as zero, and the last segment
// is simply the shorter one whose scale the pack kernel averaged over its own length.
constexpr int kYAny = 5;

// NTY: 0 for the general case; 1, 2 or 3 when Y keeps its signs and has at most 64, 128 or 192 rows
// (one tile), see below.  With Y as pieces the tile is 128 x 128 (the Y tile is three planes in LDS).
template <int XMODE, int YMODE, int NTY>
__global__ __launch_bounds__(kThreadsS) void mfma_split_gemm_kernel(const SplitArgs a)
{
    constexpr bool Y16 = YMODE == kYSign16, YP = YMODE >= kYPieces1;
    constexpr int BY = YP ? 128 : kBY;
    constexpr int kYPlane = BY * kRowBytes;
    __shared__ __attribute__((aligned(16))) unsigned char sX[2][3 * kPieceBytes];
    __shared__ __attribute__((aligned(16))) unsigned char sY[2][(YP ? 3 : 1) * kYPlane];

    // slot -> tile: consecutive slots of one XCD walk tiles in row-major (x, y) order
    const int slot = (blockIdx.x % kNumXcdS) * a.slots_per_xcd + blockIdx.x / kNumXcdS;
    if (slot >= a.tiles_total) return;
    const int x0 = (slot / a.tiles_y) * kBX, y0 = (slot % a.tiles_y) * BY;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Wave -> sub-tile of the 128 x 256 workgroup tile, as TX x TY accumulator tiles of 32 x 32.
    // General case: 2 x 4 waves of 64 x 64.  When Y has at most 64 * NTY rows the live part of the tile
    // is cut into 4 x 2 waves of 32 x (32 NTY) instead, so that all eight waves multiply (with 64 x 64
    // sub-tiles only NTY of the four wave columns would).
    // Pieces: 2 x 4 waves of 64 x 32.
    constexpr int TX = NTY == 0 ? 2 : 1, TY = YP ? 1 : NTY == 0 ? 2 : NTY;
    const int wrow0 = NTY == 0 ? (wave >> 2) * 64 : (wave & 3) * 32;
    const int wcol0 = YP ? (wave & 3) * 32 : NTY == 0 ? (wave & 3) * 64 : (wave >> 2) * (32 * NTY);
    const int nstages = (a.K + kStageK - 1) / kStageK;   // only the kXAny / kYAny pair sees a ragged K

    constexpr int kScalesPerThread = XMODE == kXScale4 ? 4 : XMODE == kXScale2 ? 2 : 1;
    constexpr int kYScalesPerThread = YMODE == kYPieces4 ? 4 : YMODE == kYPieces2 ? 2 : 1;
    struct Staged {
        float4 xr[XMODE == kXRaw ? 2 : 1];                 // raw: 2 x 4 fp32
        uint32_t xb;                                       // packed: the row's word of this stage
        float xs[kScalesPerThread];                        // packed: scales of this thread's 8 elements
        uint32_t yb;                                       // the Y row's word of this stage
        float ys[kYScalesPerThread];                       // pieces: the scales of this thread's 8 elements of Y
        uint32_t cw[XMODE == kXConv ? 8 : 1];              // conv: the word holding each element's bit
        float cs[XMODE == kXConv ? 8 : 1];                 // conv: each element's scale
        float gx[XMODE == kXAny ? 8 : 1];                  // any beta: each element's scale (or raw value)
        float gy[YMODE == kYAny ? 8 : 1];
    };

    // ---- sources (clamped, so every load below is unconditional)
    const float *xr_src[2] = {nullptr, nullptr};
    const uint32_t *xb_src = nullptr;
    const float *xs_src = nullptr;
    // packed modes: row and 8-element group of this thread.  In the conv mode the group is the same
    // for a whole wave (and lanes run along output positions), so that everything that depends on
    // k only -- channel, tap, offsets -- is computed once per wave on the scalar unit and the lanes'
    // loads fall on neighbouring activations.
    const int prow = XMODE == kXConv ? (tid & 127) : (tid >> 2);
    const int poct = XMODE == kXConv ? __builtin_amdgcn_readfirstlane(tid >> 7) : (tid & 3);
    if (XMODE == kXRaw) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int id = tid + r * kThreadsS;
            xr_src[r] = a.x_raw + (int64_t)min(x0 + (id >> 3), a.X - 1) * a.ldx_raw + (id & 7) * 4;
        }
    } else if (XMODE != kXConv) {
        const int64_t row = min(x0 + prow, a.X - 1);
        xb_src = a.x_bits + row * a.ldw_x;
        xs_src = a.x_scales + row * a.lds_x;
    }
    // conv: this thread's output position, the flat index of the window's corner, and which taps
    // fall inside the input.  (c, tap) of the thread's first element is tracked from call to call,
    // once for the loads and once for the parking; both are called for consecutive stages.
    int cv_base = 0;
    uint32_t cv_mask = 0;
    int fc0 = 0, fr0 = 0, pc0 = 0, pr0 = 0;
    if (XMODE == kXConv) {
        const int m = min(x0 + prow, a.X - 1);
        const int b = m / a.cv_ohw, pos = m - b * a.cv_ohw;
        const int oz = pos / a.cv_ow, oy = pos - oz * a.cv_ow;
        const int z0 = oz * a.cv_stride - a.cv_pad, y0w = oy * a.cv_stride - a.cv_pad;
        cv_base = (b * a.cv_c * a.cv_h + z0) * a.cv_w + y0w;
        for (int r = 0; r < a.cv_kk; ++r) {
            const int dz = r / a.cv_kw, dy = r - dz * a.cv_kw;
            const bool in = z0 + dz >= 0 && z0 + dz < a.cv_h && y0w + dy >= 0 && y0w + dy < a.cv_w;
            cv_mask |= (in ? 1u : 0u) << r;
        }
        fc0 = pc0 = (poct * 8) / a.cv_kk;
        fr0 = pr0 = (poct * 8) % a.cv_kk;
    }
    // element i (0..7) of the thread's run: its flat tensor index, forced to 0 when the tap lies
    // outside the input or past the last channel, and `keep` = all ones / zero accordingly
    auto conv_elem = [&](int c0, int r0, int i, uint32_t &e, uint32_t &keep) {
        const int t = r0 + i;
        const int cq = (t * a.cv_magic_kk) >> 16;
        const int r = t - cq * a.cv_kk;
        const int c = c0 + cq;
        const int dz = (r * a.cv_magic_kw) >> 16;
        const uint32_t taps = c < a.cv_c ? cv_mask : 0u;
        keep = (uint32_t)__builtin_amdgcn_sbfe((int)taps, (uint32_t)r, 1u);
        e = (uint32_t)(cv_base + (c * a.cv_hw + r + dz * (a.cv_w - a.cv_kw))) & keep;
    };
    auto conv_advance = [&](int &c0, int &r0) {
        c0 += a.cv_q32;
        r0 += a.cv_r32;
        if (r0 >= a.cv_kk) {
            r0 -= a.cv_kk;
            c0 += 1;
        }
    };
    // Y expansion.  Signs: thread = (row, 16-element half); pieces: thread = (row, 8-element group) like X.
    const int yrow_t = YP ? (tid >> 2) : (tid >> 1), yhalf = tid & 1, yoct = tid & 3;
    const uint32_t *yb_src = a.y_bits + (int64_t)min(y0 + yrow_t, a.Y - 1) * a.ldw_y;
    const float *ys_src = a.y_scales + (int64_t)min(y0 + yrow_t, a.Y - 1) * a.lds_y;

    auto fetch = [&](Staged &st, int stage) {
        const int sg = min(stage, nstages - 1);
        if (XMODE == kXRaw) {
#pragma unroll
            for (int r = 0; r < 2; ++r) st.xr[r] = *reinterpret_cast<const float4 *>(xr_src[r] + sg * kStageK);
        } else if (XMODE == kXConv) {
            // past the last stage c >= C: every element reads index 0 and is parked as zero
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t e, keep;
                conv_elem(fc0, fr0, i, e, keep);
                st.cw[i] = a.x_bits[e >> 5];
                st.cs[i] = a.x_scales[e >> a.log2_beta_x];
            }
            conv_advance(fc0, fr0);
        } else if constexpr (XMODE == kXAny) {
            st.xb = xb_src[sg];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t k = (uint32_t)min(sg * kStageK + poct * 8 + i, a.K - 1);
                st.gx[i] = xs_src[a.any_x_raw ? k : __umulhi(k, a.any_magic_x)];
            }
        } else {
            st.xb = xb_src[sg];
            const int sidx = (sg * kStageK + poct * 8) >> a.log2_beta_x;
#pragma unroll
            for (int j = 0; j < kScalesPerThread; ++j) st.xs[j] = xs_src[sidx + j];
        }
        st.yb = yb_src[sg];
        if constexpr (YMODE == kYAny) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t k = (uint32_t)min(sg * kStageK + yoct * 8 + i, a.K - 1);
                st.gy[i] = ys_src[__umulhi(k, a.any_magic_y)];
            }
        } else if (YP) {
            const int yidx = (sg * kStageK + yoct * 8) >> a.log2_beta_y;
#pragma unroll
            for (int j = 0; j < kYScalesPerThread; ++j) st.ys[j] = ys_src[yidx + j];
        }
    };

    // any-beta modes: 8 elements starting at k0, values +-scale (bit = 1: positive) or 0 past K
    auto any_pieces = [&](uint32_t byte, const float (&sc)[8], int k0, uint32_t sign, u32x4 &dh, u32x4 &dm, u32x4 &dl)
                          __attribute__((always_inline)) {
        uint32_t h[8], m[8], l[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t keep = k0 + i < a.K ? 0xffffffffu : 0u;
            const uint32_t minus = (~(byte >> i) << 31) & sign;
            const uint32_t value = (__builtin_bit_cast(uint32_t, sc[i]) ^ minus) & keep;
            split3(__builtin_bit_cast(float, value), h[i], m[i], l[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dh[i] = pair16(h[2 * i], h[2 * i + 1]);
            dm[i] = pair16(m[2 * i], m[2 * i + 1]);
            dl[i] = pair16(l[2 * i], l[2 * i + 1]);
        }
    };
    int park_k0 = 0;   // first k of the stage that the next call of park() handles (any-beta modes)

    auto park = [&](const Staged &st, int buf) {
        const int pk0 = park_k0;
        park_k0 += kStageK;
        if (XMODE == kXRaw) {
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int id = tid + r * kThreadsS;
                const int row = id >> 3, c = id & 7;
                uint32_t h[4], m[4], l[4];
                split3(st.xr[r].x, h[0], m[0], l[0]);
                split3(st.xr[r].y, h[1], m[1], l[1]);
                split3(st.xr[r].z, h[2], m[2], l[2]);
                split3(st.xr[r].w, h[3], m[3], l[3]);
                unsigned char *dst = &sX[buf][row * kRowBytes + c * 8];
                *reinterpret_cast<uint2 *>(dst) = make_uint2(pair16(h[0], h[1]), pair16(h[2], h[3]));
                *reinterpret_cast<uint2 *>(dst + kPieceBytes) = make_uint2(pair16(m[0], m[1]), pair16(m[2], m[3]));
                *reinterpret_cast<uint2 *>(dst + 2 * kPieceBytes) = make_uint2(pair16(l[0], l[1]), pair16(l[2], l[3]));
            }
        } else if (XMODE == kXConv) {
            uint32_t h[8], m[8], l[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                uint32_t e, keep;
                conv_elem(pc0, pr0, i, e, keep);
                // value = +-scale (bit 0 = negative), or 0 for a tap that does not exist; the pieces
                // of a negative value are the negated pieces of its magnitude
                const uint32_t minus = (~(st.cw[i] >> (e & 31)) << 31) & a.cv_sign;
                const uint32_t value = (__builtin_bit_cast(uint32_t, st.cs[i]) & keep) | minus;
                split3(__builtin_bit_cast(float, value), h[i], m[i], l[i]);
            }
            conv_advance(pc0, pr0);
            u32x4 dh, dm, dl;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                dh[i] = pair16(h[2 * i], h[2 * i + 1]);
                dm[i] = pair16(m[2 * i], m[2 * i + 1]);
                dl[i] = pair16(l[2 * i], l[2 * i + 1]);
            }
            unsigned char *dst = &sX[buf][prow * kRowBytes + poct * 16];
            *reinterpret_cast<u32x4 *>(dst) = dh;
            *reinterpret_cast<u32x4 *>(dst + kPieceBytes) = dm;
            *reinterpret_cast<u32x4 *>(dst + 2 * kPieceBytes) = dl;
        } else if constexpr (XMODE == kXAny) {
            // a raw operand carries its own sign: the mask is then 0 and the bits are ignored
            u32x4 dh, dm, dl;
            any_pieces(st.xb >> (8 * poct), st.gx, pk0 + 8 * poct, a.any_sign_x, dh, dm, dl);
            unsigned char *dst = &sX[buf][prow * kRowBytes + poct * 16];
            *reinterpret_cast<u32x4 *>(dst) = dh;
            *reinterpret_cast<u32x4 *>(dst + kPieceBytes) = dm;
            *reinterpret_cast<u32x4 *>(dst + 2 * kPieceBytes) = dl;
        } else {
            u32x4 dh, dm, dl;
            packed_pieces<kScalesPerThread>(st.xb >> (8 * poct), st.xs, dh, dm, dl);
            unsigned char *dst = &sX[buf][prow * kRowBytes + poct * 16];
            *reinterpret_cast<u32x4 *>(dst) = dh;
            *reinterpret_cast<u32x4 *>(dst + kPieceBytes) = dm;
            *reinterpret_cast<u32x4 *>(dst + 2 * kPieceBytes) = dl;
        }
        if (YP) {
            u32x4 dh, dm, dl;
            if constexpr (YMODE == kYAny)
                any_pieces(st.yb >> (8 * yoct), st.gy, pk0 + 8 * yoct, 0x80000000u, dh, dm, dl);
            else
                packed_pieces<kYScalesPerThread>(st.yb >> (8 * yoct), st.ys, dh, dm, dl);
            unsigned char *dst = &sY[buf][yrow_t * kRowBytes + yoct * 16];
            *reinterpret_cast<u32x4 *>(dst) = dh;
            *reinterpret_cast<u32x4 *>(dst + kYPlane) = dm;
            *reinterpret_cast<u32x4 *>(dst + 2 * kYPlane) = dl;
            return;
        }
        // Y: 16 signs -> 16 bf16 values +-1.0
        uint32_t ym[8];
        sign_masks<8>(~(st.yb >> (16 * yhalf)) & 0xffffu, ym);
        u32x4 y0v, y1v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            y0v[i] = ym[i] | 0x3f803f80u;
            y1v[i] = ym[4 + i] | 0x3f803f80u;
        }
        unsigned char *ydst = &sY[buf][yrow_t * kRowBytes + yhalf * 32];
        *reinterpret_cast<u32x4 *>(ydst) = y0v;
        *reinterpret_cast<u32x4 *>(ydst + 16) = y1v;
    };

    f32x16 acc[TX][TY], res[TX][TY];
#pragma unroll
    for (int p = 0; p < TX; ++p)
#pragma unroll
        for (int q = 0; q < TY; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[p][q][v] = 0.f;
                res[p][q][v] = 0.f;
            }

    // per-lane Y scale rows: the output column of accumulator tile ty is y0 + wcol0 + 32*ty + lane%32
    const float *srow[TY];
    bool col_ok[TY];
#pragma unroll
    for (int ty = 0; ty < TY; ++ty) {
        const int col = y0 + wcol0 + ty * 32 + (lane & 31);
        col_ok[ty] = col < a.Y;
        srow[ty] = a.y_scales + (int64_t)min(col, a.Y - 1) * a.lds_y;
    }

    auto apply_scale = [&](const float (&sc)[TY]) {
#pragma unroll
        for (int tx = 0; tx < TX; ++tx)
#pragma unroll
            for (int ty = 0; ty < TY; ++ty)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    res[tx][ty][v] = __builtin_fmaf(sc[ty], acc[tx][ty][v], res[tx][ty][v]);
                    acc[tx][ty][v] = 0.f;
                }
    };

    float sc_seg[TY] = {};
    // One K stage: multiply the tile parked in LDS buffer (stage mod 2), request stage + 3 into
    // `incoming`, and park `ready` (stage + 1, requested three stages ago) in the other buffer.
    auto run_stage = [&](int stage, const Staged &ready, Staged &incoming) {
        const int buf = stage & 1;
        if (YP) {
            // both operands as pieces: the six piece pairs that matter, smallest contributions first
            // (hi,lo) (lo,hi) (mid,mid) (hi,mid) (mid,hi) (hi,hi); what is dropped is below 2^-24 of a term
            fetch(incoming, stage + 3);
            const unsigned char *pxp = &sX[buf][(wrow0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
            const unsigned char *pyp = &sY[buf][(wcol0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
#pragma unroll
            for (int ks = 0; ks < kStageK / 16; ++ks) {
                bf16x8 fxp[3][TX], fyp[3];
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    fyp[p] = *reinterpret_cast<const bf16x8 *>(pyp + p * kYPlane + ks * 32);
#pragma unroll
                    for (int tx = 0; tx < TX; ++tx)
                        fxp[p][tx] = *reinterpret_cast<const bf16x8 *>(pxp + p * kPieceBytes + tx * 32 * kRowBytes + ks * 32);
                }
#pragma unroll
                for (int q = 0; q < 6; ++q)
#pragma unroll
                    for (int tx = 0; tx < TX; ++tx)
                        res[tx][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fxp[kPiecePairs[q][0]][tx], fyp[kPiecePairs[q][1]], res[tx][0], 0, 0, 0);
            }
            park(ready, buf ^ 1);
            __syncthreads();
            return;
        }
        // The scales are requested before the prefetch: loads return in order, so waiting for the
        // scales at the end of the stage then leaves the prefetch in flight.
        float sc16[2][TY];
        bool seg_last = false;
        if (Y16) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int ty = 0; ty < TY; ++ty) sc16[ks][ty] = srow[ty][stage * 2 + ks];
        } else {
            // stages per Y segment is a power of two.  The scale is re-read every stage rather than
            // at segment starts only: a load under a condition hides the number of outstanding loads
            // from the compiler, which then waits for all of them, prefetches included.
            seg_last = ((stage + 1) & (a.stages_per_yseg - 1)) == 0;
#pragma unroll
            for (int ty = 0; ty < TY; ++ty) sc_seg[ty] = srow[ty][stage >> a.log2_stages_per_yseg];
        }
        fetch(incoming, stage + 3);
        const unsigned char *px = &sX[buf][(wrow0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
        const unsigned char *py = &sY[buf][(wcol0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
#pragma unroll
        for (int ks = 0; ks < kStageK / 16; ++ks) {
            bf16x8 fy[TY];
#pragma unroll
            for (int ty = 0; ty < TY; ++ty)
                fy[ty] = *reinterpret_cast<const bf16x8 *>(py + ty * 32 * kRowBytes + ks * 32);
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                bf16x8 fx[TX];
#pragma unroll
                for (int tx = 0; tx < TX; ++tx)
                    fx[tx] = *reinterpret_cast<const bf16x8 *>(px + p * kPieceBytes + tx * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int tx = 0; tx < TX; ++tx)
#pragma unroll
                    for (int ty = 0; ty < TY; ++ty)
                        acc[tx][ty] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[tx], fy[ty], acc[tx][ty], 0, 0, 0);
            }
            if (Y16) apply_scale(sc16[ks]);
        }
        // The next stage is parked before the (conditional) segment epilogue so that the splitting
        // and sign-expansion arithmetic sits in the same scheduling region as the MFMAs.
        park(ready, buf ^ 1);   // past the last stage this parks data that nobody reads
        if (!Y16 && seg_last) apply_scale(sc_seg);
        __syncthreads();
    };

    Staged s0, s1, s2;
    fetch(s0, 0);
    park(s0, 0);
    fetch(s0, 1);
    fetch(s1, 2);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 3) {
        run_stage(stage, s0, s2);
        if (stage + 1 < nstages) run_stage(stage + 1, s1, s0);
        if (stage + 2 < nstages) run_stage(stage + 2, s2, s1);
    }

    if (XMODE == kXConv) {
        // Output is B x Y x OH x OW: positions are contiguous, filters are OH*OW apart.  The
        // accumulator tiles hold filters across lanes, so each 32 x 32 tile is turned through LDS
        // (row stride 33 words) and written with positions across lanes.
        __syncthreads();   // every wave has finished reading the operand tiles
        float *turn = reinterpret_cast<float *>(&sX[0][0]) + wave * (32 * 33);
#pragma unroll
        for (int tx = 0; tx < TX; ++tx) {
            const int m = x0 + wrow0 + tx * 32 + (lane & 31);
            const int mc = min(m, a.X - 1);
            const int b = mc / a.cv_ohw, pos = mc - b * a.cv_ohw;
            float *dst = a.out + (int64_t)b * a.Y * a.cv_ohw + pos;
#pragma unroll
            for (int ty = 0; ty < TY; ++ty) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    turn[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * 33 + (lane & 31)] = res[tx][ty][v];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int cl = 2 * j + (lane >> 5);
                    const int col = y0 + wcol0 + ty * 32 + cl;
                    const float val = turn[(lane & 31) * 33 + cl];
                    if (m < a.X && col < a.Y) dst[(int64_t)col * a.cv_ohw] = val;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        return;
    }
#pragma unroll
    for (int tx = 0; tx < TX; ++tx)
#pragma unroll
        for (int ty = 0; ty < TY; ++ty) {
            if (!col_ok[ty]) continue;
            const int col = y0 + wcol0 + ty * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = x0 + wrow0 + tx * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.X) a.out[(int64_t)row * a.ld_out_x + (int64_t)col * a.ld_out_y] = res[tx][ty][v];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Convolution layer with the activations staged once per workgroup.
//
// The conv mode of mfma_split_gemm_kernel builds every element of the (positions x taps) operand
// from memory, i.e. each activation KH*KW times.  Here a workgroup owns R whole output rows of one
// image (R * OW <= 128 positions) and keeps, for the channels the current K stages touch, the
// input patch those rows need -- ((R - 1) * stride + KH) rows x (W + 2 pad) columns, zero outside
// the image -- in LDS as three planes of bf16 pieces (the exact split of +-scale, done once per
// activation).  Channels live in a ring of NS slots.  The 128 x 32 operand tile of a stage is then
// gathered LDS -> LDS: element (m, k) sits at
//     slot(c) * PS + (orow * stride + dz) * PW + oy * stride + dy
// = a per-position part (fixed per thread) + a per-k part (one table of 32 entries per stage,
// written by 32 threads a stage ahead).  From there on -- fragment reads, MFMAs, filter scale per
// segment, turned store -- it is the kernel above.
//
// Schedule of stage s (one barrier per stage): multiply tile s; gather tile s + 1 from the patch;
// turn the loads requested two stages ago into the patch planes of the channels that stage s + 2
// brings in, and expand the filter words of stage s + 1; write the k table of stage s + 2; request
// the loads of stage s + 4.  A slot is overwritten only by a channel NS further on, and NS exceeds
// the channel span of two consecutive stages, so the gather never reads a slot being rewritten.
constexpr int kPatchPlane = 8192;           // bf16 elements per piece plane (16 KB)

struct ConvPatchArgs {
    const uint32_t *x_bits;
    const float *x_scales;
    const uint32_t *y_bits;
    const float *y_scales;
    float *out;
    int32_t ldw_y, lds_y;
    int32_t Y, K;
    int32_t log2_beta_x, stages_per_yseg, log2_stages_per_yseg;
    int32_t C, H, W, HW, OH, OW, OHW, KW, KK, stride, pad;
    int32_t R, tiles_per_image, tiles_y, tiles_total, slots_per_xcd;
    int32_t PW, P, PS, NS;
    int32_t nch;                 // most channels a stage can bring in: ceil(32 / KK)
    uint32_t sign;               // 0x80000000; 0 when the tensor is unquantised (see launch_mfma_split_conv)
    uint32_t last_elem;          // B*C*H*W - 1
    int32_t q32, r32, magic_kw;
};

// IPT: (channel, patch element) items a thread stages per stage; IPT * 512 >= nch * P.
template <int IPT, bool Y16, int NTY>
__global__ __launch_bounds__(kThreadsS) void conv_patch_kernel(const ConvPatchArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char sX[2][3 * kPieceBytes];
    __shared__ __attribute__((aligned(16))) unsigned char sY[2][kBY * kRowBytes];
    __shared__ __attribute__((aligned(16))) unsigned short sPatch[3][kPatchPlane];
    __shared__ __attribute__((aligned(16))) uint32_t sKoff[4][kStageK];

    const int slot_id = (blockIdx.x % kNumXcdS) * a.slots_per_xcd + blockIdx.x / kNumXcdS;
    if (slot_id >= a.tiles_total) return;
    // (a tile covers 256 filters, or 64 NTY of them: the latter also with several tiles along the filters,
    // which the launcher uses to fill the chip when there are few position tiles)
    const int tile_x = slot_id / a.tiles_y, y0 = (slot_id % a.tiles_y) * (NTY == 0 ? kBY : 64 * NTY);
    const int img = tile_x / a.tiles_per_image, oz0 = (tile_x % a.tiles_per_image) * a.R;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // wave -> sub-tile, as in mfma_split_gemm_kernel
    constexpr int TX = NTY == 0 ? 2 : 1, TY = NTY == 0 ? 2 : NTY;
    const int wrow0 = NTY == 0 ? (wave >> 2) * 64 : (wave & 3) * 32;
    const int wcol0 = NTY == 0 ? (wave & 3) * 64 : (wave >> 2) * (32 * NTY);
    const int nstages = a.K / kStageK;
    const int npos = a.R * a.OW;                            // positions of a full tile (<= 128)

    // ---- role 1: owner of IPT staging items.  Item i = tid + 512 j is patch element (i mod P) of the
    // (i div P)-th channel a stage brings in; the same items every stage.
    uint32_t pe0[IPT], pkeep[IPT];
    int pch[IPT], pat[IPT];
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
        const int item = tid + j * kThreadsS;
        const int ch = item / a.P, p = item - ch * a.P;
        const int prow = p / a.PW, pcol = p - prow * a.PW;
        const int z = oz0 * a.stride - a.pad + prow, y = pcol - a.pad;
        const bool inside = z >= 0 && z < a.H && y >= 0 && y < a.W;
        pch[j] = ch;                                   // >= nch: the item does not exist
        pat[j] = p;
        pkeep[j] = inside ? 0xffffffffu : 0u;
        pe0[j] = inside ? (uint32_t)((img * a.C * a.H + z) * a.W + y) + (uint32_t)(ch * a.HW) : 0u;
    }
    // ---- role 2: gatherer of 8 consecutive k of one position
    const int grow = tid & 127, goct = __builtin_amdgcn_readfirstlane(tid >> 7);
    uint32_t gbase;   // byte offset of the position's window corner inside a patch slot
    {
        const int ml = min(grow, npos - 1);
        const int orow = ml / a.OW, oy = ml - orow * a.OW;
        gbase = (uint32_t)((orow * a.stride) * a.PW + oy * a.stride) * 2u;
    }
    // ---- role 3: expander of 16 filter signs
    const int yrow_t = tid >> 1, yhalf = tid & 1;
    const uint32_t *yb_src = a.y_bits + (int64_t)min(y0 + yrow_t, a.Y - 1) * a.ldw_y;

    struct Staged {
        uint32_t pw[IPT];
        float ps[IPT];
        uint32_t yb;
    };
    const char *xb_bytes = reinterpret_cast<const char *>(a.x_bits);
    const char *xs_bytes = reinterpret_cast<const char *>(a.x_scales);

    // Channels that stage sx brings in: (last channel of stage sx - 1, last channel of stage sx].
    // Both walkers are advanced once per call, and the calls come in stage order.
    struct Walker {
        int q, r, prev;   // (32 sx + 31) div / mod KK, and the last channel of the previous stage
    };
    Walker fwalk{31 / a.KK, 31 % a.KK, -1}, pwalk{31 / a.KK, 31 % a.KK, -1};
    int pslot = 0;        // ring slot of the first channel the next park brings in
    auto advance = [&](Walker &w, int last) {
        w.prev = last;
        w.q += a.q32;
        w.r += a.r32;
        if (w.r >= a.KK) {
            w.r -= a.KK;
            w.q += 1;
        }
    };

    auto fetch = [&](Staged &st, int sx) {
        const int last = min(fwalk.q, a.C - 1);
        const uint32_t first_off = (uint32_t)((fwalk.prev + 1) * a.HW);
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            // unconditional loads; an item whose channel lies past the stage's (or the tensor's) last
            // one reads a clamped index and is not parked
            const uint32_t e = min((pe0[j] + first_off) & pkeep[j], a.last_elem);
            st.pw[j] = *reinterpret_cast<const uint32_t *>(xb_bytes + ((e >> 5) << 2));
            st.ps[j] = *reinterpret_cast<const float *>(xs_bytes + ((e >> a.log2_beta_x) << 2));
        }
        st.yb = yb_src[min(max(sx - 1, 0), nstages - 1)];
        advance(fwalk, last);
    };

    const bool yrow_live = y0 + yrow_t < a.Y;
    auto park = [&](const Staged &st, int sx) {
        const int last = min(pwalk.q, a.C - 1);
        const int nnew = last - pwalk.prev;
        const uint32_t first_off = (uint32_t)((pwalk.prev + 1) * a.HW);
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            const uint32_t e = (pe0[j] + first_off) & pkeep[j];
            const uint32_t minus = (~(st.pw[j] >> (e & 31)) << 31) & a.sign;
            const uint32_t value = (__builtin_bit_cast(uint32_t, st.ps[j]) & pkeep[j]) | minus;
            uint32_t h, m, l;
            split3(__builtin_bit_cast(float, value), h, m, l);
            if (pch[j] < nnew) {
                int slot = pslot + pch[j];
                slot -= slot >= a.NS ? a.NS : 0;
                const int at = slot * a.PS + pat[j];
                sPatch[0][at] = (unsigned short)(h >> 16);
                sPatch[1][at] = (unsigned short)(m >> 16);
                sPatch[2][at] = (unsigned short)(l >> 16);
            }
        }
        pslot += nnew;
        pslot -= pslot >= a.NS ? a.NS : 0;
        advance(pwalk, last);
        // filter signs of stage sx - 1 -> +-1.0 (rows past Y are never multiplied into a stored column)
        if (yrow_live) {
            const int ybuf = max(sx - 1, 0) & 1;
            uint32_t ym[8];
            sign_masks<8>(~(st.yb >> (16 * yhalf)) & 0xffffu, ym);
            u32x4 y0v, y1v;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                y0v[i] = ym[i] | 0x3f803f80u;
                y1v[i] = ym[4 + i] | 0x3f803f80u;
            }
            unsigned char *ydst = &sY[ybuf][yrow_t * kRowBytes + yhalf * 32];
            *reinterpret_cast<u32x4 *>(ydst) = y0v;
            *reinterpret_cast<u32x4 *>(ydst + 16) = y1v;
        }
    };

    // k table: thread t < 32 follows k = 32 j + t through the stages
    int tslot = (tid / a.KK) % a.NS, tr = tid % a.KK;   // ring slot of the channel, tap
    auto write_table = [&](int j) {
        if (tid < kStageK) {
            const int dz = (tr * a.magic_kw) >> 16, dy = tr - dz * a.KW;
            sKoff[j & 3][tid] = (uint32_t)(tslot * a.PS + dz * a.PW + dy) * 2u;
            tslot += a.q32;
            tr += a.r32;
            if (tr >= a.KK) {
                tr -= a.KK;
                tslot += 1;
            }
            tslot -= tslot >= a.NS ? a.NS : 0;   // q32 + 1 < NS: one step back is enough
        }
    };

    auto gather = [&](int j) {
        const u32x4 *tab = reinterpret_cast<const u32x4 *>(&sKoff[j & 3][goct * 8]);
        const u32x4 t0 = tab[0], t1 = tab[1];
        const uint32_t off[8] = {t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
        const unsigned char *plane = reinterpret_cast<const unsigned char *>(&sPatch[0][0]);
        unsigned char *dst = &sX[j & 1][grow * kRowBytes + goct * 16];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            uint32_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = *reinterpret_cast<const unsigned short *>(plane + p * (kPatchPlane * 2) + gbase + off[i]);
            u32x4 d;
#pragma unroll
            for (int i = 0; i < 4; ++i) d[i] = v[2 * i] | (v[2 * i + 1] << 16);
            *reinterpret_cast<u32x4 *>(dst + p * kPieceBytes) = d;
        }
    };

    f32x16 acc[TX][TY], res[TX][TY];
#pragma unroll
    for (int p = 0; p < TX; ++p)
#pragma unroll
        for (int q = 0; q < TY; ++q)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[p][q][v] = 0.f;
                res[p][q][v] = 0.f;
            }
    const float *srow[TY];
#pragma unroll
    for (int ty = 0; ty < TY; ++ty)
        srow[ty] = a.y_scales + (int64_t)min(y0 + wcol0 + ty * 32 + (lane & 31), a.Y - 1) * a.lds_y;
    auto apply_scale = [&](const float (&sc)[TY]) {
#pragma unroll
        for (int tx = 0; tx < TX; ++tx)
#pragma unroll
            for (int ty = 0; ty < TY; ++ty)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    res[tx][ty][v] = __builtin_fmaf(sc[ty], acc[tx][ty][v], res[tx][ty][v]);
                    acc[tx][ty][v] = 0.f;
                }
    };

    float sc_seg[TY] = {};
    auto run_stage = [&](int stage, const Staged &ready, Staged &incoming) {
        const int buf = stage & 1;
        // The scales are requested before the prefetch: loads return in order, so waiting for the
        // scales at the end of the stage then leaves the prefetch in flight.
        float sc16[2][TY];
        bool seg_last = false;
        if (Y16) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int ty = 0; ty < TY; ++ty) sc16[ks][ty] = srow[ty][stage * 2 + ks];
        } else {
            // stages per Y segment is a power of two.  The scale is re-read every stage rather than
            // at segment starts only: a load under a condition hides the number of outstanding loads
            // from the compiler, which then waits for all of them, prefetches included.
            seg_last = ((stage + 1) & (a.stages_per_yseg - 1)) == 0;
#pragma unroll
            for (int ty = 0; ty < TY; ++ty) sc_seg[ty] = srow[ty][stage >> a.log2_stages_per_yseg];
        }
        fetch(incoming, stage + 4);
        const unsigned char *px = &sX[buf][(wrow0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
        const unsigned char *py = &sY[buf][(wcol0 + (lane & 31)) * kRowBytes + (lane >> 5) * 16];
#pragma unroll
        for (int ks = 0; ks < kStageK / 16; ++ks) {
            bf16x8 fy[TY];
#pragma unroll
            for (int ty = 0; ty < TY; ++ty)
                fy[ty] = *reinterpret_cast<const bf16x8 *>(py + ty * 32 * kRowBytes + ks * 32);
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                bf16x8 fx[TX];
#pragma unroll
                for (int tx = 0; tx < TX; ++tx)
                    fx[tx] = *reinterpret_cast<const bf16x8 *>(px + p * kPieceBytes + tx * 32 * kRowBytes + ks * 32);
#pragma unroll
                for (int tx = 0; tx < TX; ++tx)
#pragma unroll
                    for (int ty = 0; ty < TY; ++ty)
                        acc[tx][ty] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[tx], fy[ty], acc[tx][ty], 0, 0, 0);
            }
            if (Y16) apply_scale(sc16[ks]);
        }
        gather(stage + 1);
        park(ready, stage + 2);
        write_table(stage + 2);
        if (!Y16 && seg_last) apply_scale(sc_seg);
        __syncthreads();
    };

    Staged s0, s1, s2;
    fetch(s0, 0);
    fetch(s1, 1);
    write_table(0);
    write_table(1);
    park(s0, 0);
    park(s1, 1);
    __syncthreads();
    fetch(s0, 2);
    fetch(s1, 3);
    gather(0);
    __syncthreads();
    for (int stage = 0; stage < nstages; stage += 3) {
        run_stage(stage, s0, s2);
        if (stage + 1 < nstages) run_stage(stage + 1, s1, s0);
        if (stage + 2 < nstages) run_stage(stage + 2, s2, s1);
    }

    // ---- store: out is B x Y x OH x OW; each 32 x 32 accumulator tile is turned through LDS so that
    // lanes run along positions
    // (the loop's last barrier has passed; the turn areas are per wave, inside sX, which nobody
    // multiplies from any more)
    float *turn = reinterpret_cast<float *>(&sX[0][0]) + wave * (32 * 33);
#pragma unroll
    for (int tx = 0; tx < TX; ++tx) {
        const int ml = wrow0 + tx * 32 + (lane & 31);
        const int mc = min(ml, npos - 1);
        const int orow = mc / a.OW, oy = mc - orow * a.OW;
        const bool pos_ok = ml < npos && oz0 + orow < a.OH;
        float *dst = a.out + ((int64_t)img * a.Y * a.OH + (oz0 + orow)) * a.OW + oy;
#pragma unroll
        for (int ty = 0; ty < TY; ++ty) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                turn[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * 33 + (lane & 31)] = res[tx][ty][v];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int cl = 2 * j + (lane >> 5);
                const int col = y0 + wcol0 + ty * 32 + cl;
                const float val = turn[(lane & 31) * 33 + cl];
                if (pos_ok && col < a.Y) dst[(int64_t)col * a.OHW] = val;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

template <int XMODE>
hipError_t launch_mode(const SplitArgs &a, int beta_y, unsigned grid, hipStream_t s)
{
    const dim3 g(grid), b(kThreadsS);
    if (beta_y < 16) {
        // a Y segment shorter than an MFMA step: Y as pieces
        if (beta_y == 2)
            mfma_split_gemm_kernel<XMODE, kYPieces4, 0><<<g, b, 0, s>>>(a);
        else if (beta_y == 4)
            mfma_split_gemm_kernel<XMODE, kYPieces2, 0><<<g, b, 0, s>>>(a);
        else
            mfma_split_gemm_kernel<XMODE, kYPieces1, 0><<<g, b, 0, s>>>(a);
        return hipGetLastError();
    }
    const int nty = a.Y <= 64 ? 1 : a.Y <= 128 ? 2 : a.Y <= 192 ? 3 : 0;
#define HBMM_SPLIT_LAUNCH(YM)                                                                        \
    do {                                                                                             \
        if (nty == 1)                                                                                \
            mfma_split_gemm_kernel<XMODE, YM, 1><<<g, b, 0, s>>>(a);                                 \
        else if (nty == 2)                                                                           \
            mfma_split_gemm_kernel<XMODE, YM, 2><<<g, b, 0, s>>>(a);                                 \
        else if (nty == 3)                                                                           \
            mfma_split_gemm_kernel<XMODE, YM, 3><<<g, b, 0, s>>>(a);                                 \
        else                                                                                         \
            mfma_split_gemm_kernel<XMODE, YM, 0><<<g, b, 0, s>>>(a);                                 \
    } while (0)
    if (beta_y == 16)
        HBMM_SPLIT_LAUNCH(kYSign16);
    else
        HBMM_SPLIT_LAUNCH(kYSign);
#undef HBMM_SPLIT_LAUNCH
    return hipGetLastError();
}

int ilog2s(int v)
{
    int s = 0;
    while ((1 << s) < v) ++s;
    return s;
}

}  // namespace

hipError_t launch_mfma_split_gemm(const SplitGemmOperand &x, const SplitGemmOperand &y, int64_t K, float *out,
                                  int64_t ld_out_x, int64_t ld_out_y, hipStream_t s)
{
    // x: dense side (beta 1 = raw fp32 through x.raw, or packed with any supported beta)
    // y: packed; beta >= 16 keeps its signs, a shorter segment is rebuilt as fp32 values like x
    if (y.beta < 2 || y.bits == nullptr || K % kStageK != 0) return hipErrorNotSupported;
    if (x.beta == 1 && (x.raw == nullptr || x.ld_raw % 4 != 0)) return hipErrorNotSupported;
    if (x.beta != 1 && x.bits == nullptr) return hipErrorNotSupported;
    SplitArgs a{};
    a.x_raw = x.raw; a.ldx_raw = x.ld_raw;
    a.x_bits = x.bits; a.x_scales = x.scales; a.ldw_x = (int32_t)x.ldw; a.lds_x = (int32_t)x.lds;
    a.y_bits = y.bits; a.y_scales = y.scales; a.ldw_y = (int32_t)y.ldw; a.lds_y = (int32_t)y.lds;
    a.out = out; a.ld_out_x = ld_out_x; a.ld_out_y = ld_out_y;
    a.X = (int32_t)x.rows; a.Y = (int32_t)y.rows; a.K = (int32_t)K;
    a.log2_beta_x = ilog2s(x.beta);
    a.log2_beta_y = ilog2s(y.beta);
    a.stages_per_yseg = y.beta >= 32 ? y.beta / kStageK : 1;
    a.log2_stages_per_yseg = ilog2s(a.stages_per_yseg);
    const int by = y.beta < 16 ? 128 : kBY;
    const int64_t tiles_x = (x.rows + kBX - 1) / kBX, tiles_y = (y.rows + by - 1) / by;
    const int64_t total = tiles_x * tiles_y;
    const int64_t per_xcd = (total + kNumXcdS - 1) / kNumXcdS;
    if (per_xcd * kNumXcdS > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.tiles_y = (int32_t)tiles_y; a.tiles_total = (int32_t)total; a.slots_per_xcd = (int32_t)per_xcd;
    const unsigned grid = (unsigned)(per_xcd * kNumXcdS);
    if (x.beta == 1) return launch_mode<kXRaw>(a, y.beta, grid, s);
    if (x.beta == 2) return launch_mode<kXScale4>(a, y.beta, grid, s);
    if (x.beta == 4) return launch_mode<kXScale2>(a, y.beta, grid, s);
    return launch_mode<kXScale1>(a, y.beta, grid, s);
}

hipError_t launch_mfma_split_any(const SplitGemmOperand &x, const SplitGemmOperand &y, int64_t K, float *out,
                                 int64_t ld_out_x, int64_t ld_out_y, hipStream_t s)
{
    if (y.beta < 2 || y.beta > 256 || y.bits == nullptr || y.scales == nullptr) return hipErrorNotSupported;
    if (x.beta < 1 || x.beta > 256 || K < 1 || K >= (1 << 24)) return hipErrorNotSupported;
    if (x.beta == 1 ? x.raw == nullptr : (x.bits == nullptr || x.scales == nullptr)) return hipErrorNotSupported;
    const bool raw = x.beta == 1;
    if ((raw ? x.ld_raw : x.ldw) > 0x7fffffffLL || x.lds > 0x7fffffffLL) return hipErrorNotSupported;
    SplitArgs a{};
    // raw X: the "scales" are the values; the word loaded as bits is any in-bounds word of the row
    a.x_bits = raw ? reinterpret_cast<const uint32_t *>(x.raw) : x.bits;
    a.x_scales = raw ? x.raw : x.scales;
    a.ldw_x = (int32_t)(raw ? x.ld_raw : x.ldw);
    a.lds_x = (int32_t)(raw ? x.ld_raw : x.lds);
    a.any_x_raw = raw ? 1 : 0;
    a.any_sign_x = raw ? 0u : 0x80000000u;
    a.any_magic_x = raw ? 0u : (uint32_t)(((1ull << 32) + x.beta - 1) / x.beta);
    a.any_magic_y = (uint32_t)(((1ull << 32) + y.beta - 1) / y.beta);
    a.y_bits = y.bits; a.y_scales = y.scales; a.ldw_y = (int32_t)y.ldw; a.lds_y = (int32_t)y.lds;
    a.out = out; a.ld_out_x = ld_out_x; a.ld_out_y = ld_out_y;
    a.X = (int32_t)x.rows; a.Y = (int32_t)y.rows; a.K = (int32_t)K;
    const int64_t tiles_x = (x.rows + kBX - 1) / kBX, tiles_y = (y.rows + 127) / 128;
    const int64_t total = tiles_x * tiles_y;
    const int64_t per_xcd = (total + kNumXcdS - 1) / kNumXcdS;
    if (per_xcd * kNumXcdS > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.tiles_y = (int32_t)tiles_y; a.tiles_total = (int32_t)total; a.slots_per_xcd = (int32_t)per_xcd;
    mfma_split_gemm_kernel<kXAny, kYAny, 0><<<dim3((unsigned)(per_xcd * kNumXcdS)), dim3(kThreadsS), 0, s>>>(a);
    return hipGetLastError();
}

// The staged-patch kernel when the layer fits it; false = use the gather kernel.
static bool try_launch_conv_patch(const ConvActivations &x, const SplitGemmOperand &y, const ConvGeometry &g, int64_t OH,
                                  int64_t OW, float *out, hipStream_t s, hipError_t &err)
{
    const int KK = g.KH * g.KW;
    if (OW > 128 || KK < 2) return false;
    if (y.beta == 16) return false;   // the per-16 epilogue's registers do not fit next to the staging
    int R = (int)(128 / OW < OH ? 128 / OW : OH);
    const int tiles_per_image = (int)((OH + R - 1) / R);
    R = (int)((OH + tiles_per_image - 1) / tiles_per_image);
    const int PW = (int)g.W + 2 * g.pad, PR = (R - 1) * g.stride + g.KH, P = PR * PW;
    const int nch = (kStageK + KK - 1) / KK;
    const int ipt = (nch * P + kThreadsS - 1) / kThreadsS;
    if (ipt > 8) return false;
    const int NS = (2 * kStageK - 1) / KK + 3, PS = (P + 7) / 8 * 8;
    if (NS * PS > kPatchPlane) return false;
    // Filters per tile: 256, or all of them when there are at most 192; narrower tiles (128, then 64
    // filters: every position tile is then staged by several workgroups) as long as the grid does not
    // give every compute unit a workgroup.
    int nty = y.rows <= 64 ? 1 : y.rows <= 128 ? 2 : y.rows <= 192 ? 3 : 0;
    const int64_t tiles_x = g.B * tiles_per_image;
    auto tiles_along_y = [&](int n) { return (y.rows + (n == 0 ? kBY : 64 * n) - 1) / (n == 0 ? kBY : 64 * n); };
    if (nty == 0 && tiles_x * tiles_along_y(0) < 256) nty = 2;
    if (nty == 2 && y.rows > 64 && tiles_x * tiles_along_y(2) < 256) nty = 1;
    const int64_t tiles_y = tiles_along_y(nty);
    const int64_t total = tiles_x * tiles_y, per_xcd = (total + kNumXcdS - 1) / kNumXcdS;
    if (per_xcd * kNumXcdS > 0x7fffffffLL) return false;
    ConvPatchArgs a{};
    // beta = 1: `scales` is the unquantised tensor.  It then plays both parts: read as the "scale" of
    // element e (segment length 1) it is the value itself, sign included, and the sign taken from the
    // bit word is switched off; the word loads still happen and are pointed at the same memory.
    a.x_bits = x.beta == 1 ? reinterpret_cast<const uint32_t *>(x.scales) : x.bits;
    a.x_scales = x.scales; a.log2_beta_x = ilog2s(x.beta); a.sign = x.beta == 1 ? 0u : 0x80000000u;
    a.y_bits = y.bits; a.y_scales = y.scales; a.ldw_y = (int32_t)y.ldw; a.lds_y = (int32_t)y.lds;
    a.out = out; a.Y = (int32_t)y.rows; a.K = (int32_t)(g.C * KK);
    a.stages_per_yseg = y.beta >= 32 ? y.beta / kStageK : 1;
    a.log2_stages_per_yseg = ilog2s(a.stages_per_yseg);
    a.C = (int32_t)g.C; a.H = (int32_t)g.H; a.W = (int32_t)g.W; a.HW = (int32_t)(g.H * g.W);
    a.OH = (int32_t)OH; a.OW = (int32_t)OW; a.OHW = (int32_t)(OH * OW);
    a.KW = g.KW; a.KK = KK; a.stride = g.stride; a.pad = g.pad;
    a.R = R; a.tiles_per_image = tiles_per_image; a.tiles_y = (int32_t)tiles_y; a.tiles_total = (int32_t)total;
    a.slots_per_xcd = (int32_t)per_xcd;
    a.PW = PW; a.P = P; a.PS = PS; a.NS = NS; a.nch = nch;
    a.last_elem = (uint32_t)(g.B * g.C * g.H * g.W - 1);
    a.q32 = kStageK / KK; a.r32 = kStageK % KK; a.magic_kw = 65536 / g.KW + 1;
    const dim3 grid((unsigned)(per_xcd * kNumXcdS)), block(kThreadsS);
#define HBMM_PATCH_LAUNCH(I)                                                \
    do {                                                                    \
        if (nty == 1)                                                       \
            conv_patch_kernel<I, false, 1><<<grid, block, 0, s>>>(a);       \
        else if (nty == 2)                                                  \
            conv_patch_kernel<I, false, 2><<<grid, block, 0, s>>>(a);       \
        else if (nty == 3)                                                  \
            conv_patch_kernel<I, false, 3><<<grid, block, 0, s>>>(a);       \
        else                                                                \
            conv_patch_kernel<I, false, 0><<<grid, block, 0, s>>>(a);       \
    } while (0)
    if (ipt <= 2)
        HBMM_PATCH_LAUNCH(2);
    else if (ipt <= 4)
        HBMM_PATCH_LAUNCH(4);
    else if (ipt <= 6)
        HBMM_PATCH_LAUNCH(6);
    else
        HBMM_PATCH_LAUNCH(8);
#undef HBMM_PATCH_LAUNCH
    err = hipGetLastError();
    return true;
}

hipError_t launch_mfma_split_conv(const ConvActivations &x, const SplitGemmOperand &y, const ConvGeometry &g, float *out,
                                  hipStream_t s)
{
    const int64_t OH = (g.H + 2 * g.pad - g.KH) / g.stride + 1, OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
    const int64_t K = g.C * g.KH * g.KW, M = g.B * OH * OW;
    if (y.beta < 2 || y.bits == nullptr || K % kStageK != 0 || g.KH * g.KW > 32) return hipErrorNotSupported;
    if (g.B * g.C * g.H * g.W > 0x7fffffffLL || M > 0x7fffffffLL) return hipErrorNotSupported;
    const bool y_pieces = y.beta < 16;   // a filter segment shorter than an MFMA step: filters rebuilt as fp32 values
    if (g.algo != 1 && !y_pieces) {
        hipError_t err = hipSuccess;
        if (try_launch_conv_patch(x, y, g, OH, OW, out, s, err)) return err;
    }
    SplitArgs a{};
    a.x_bits = x.beta == 1 ? reinterpret_cast<const uint32_t *>(x.scales) : x.bits;   // as in the patch kernel
    a.x_scales = x.scales; a.log2_beta_x = ilog2s(x.beta); a.cv_sign = x.beta == 1 ? 0u : 0x80000000u;
    a.y_bits = y.bits; a.y_scales = y.scales; a.ldw_y = (int32_t)y.ldw; a.lds_y = (int32_t)y.lds;
    a.out = out;
    a.X = (int32_t)M; a.Y = (int32_t)y.rows; a.K = (int32_t)K;
    a.log2_beta_y = ilog2s(y.beta);
    a.stages_per_yseg = y.beta >= 32 ? y.beta / kStageK : 1;
    a.log2_stages_per_yseg = ilog2s(a.stages_per_yseg);
    a.cv_c = (int32_t)g.C; a.cv_h = (int32_t)g.H; a.cv_w = (int32_t)g.W; a.cv_hw = (int32_t)(g.H * g.W);
    a.cv_ow = (int32_t)OW; a.cv_ohw = (int32_t)(OH * OW);
    a.cv_kw = g.KW; a.cv_kk = g.KH * g.KW; a.cv_stride = g.stride; a.cv_pad = g.pad;
    a.cv_magic_kk = 65536 / a.cv_kk + 1; a.cv_magic_kw = 65536 / a.cv_kw + 1;
    a.cv_q32 = kStageK / a.cv_kk; a.cv_r32 = kStageK % a.cv_kk;
    const int by = y_pieces ? 128 : kBY;
    const int64_t tiles_x = (M + kBX - 1) / kBX, tiles_y = (y.rows + by - 1) / by;
    const int64_t total = tiles_x * tiles_y;
    const int64_t per_xcd = (total + kNumXcdS - 1) / kNumXcdS;
    if (per_xcd * kNumXcdS > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.tiles_y = (int32_t)tiles_y; a.tiles_total = (int32_t)total; a.slots_per_xcd = (int32_t)per_xcd;
    return launch_mode<kXConv>(a, y.beta, (unsigned)(per_xcd * kNumXcdS), s);
}

}  // namespace hbmm
