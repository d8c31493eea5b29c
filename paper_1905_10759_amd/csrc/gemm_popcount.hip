// XNOR + popcount HBMM (HadaNets Eq. 7) on the gfx950 vector ALU, with the fp32 block-scale
// epilogue fused in.
//
// For one output and one segment g of G = min(beta_p, beta_q) bits,
//     d = sum_k (+-1)(+-1) = G - 2 * popcount(p_word xor q_word)
// (Eq. 7 prints popcount(xnor(.)), the count of agreeing signs; d is the signed count it stands
// for), and the output accumulates  sP * sQ * d  in fp32, in ascending g.
//
// Mapping to the machine.  The cost is two VALU instructions per 32 binary multiply-adds
// (v_xor_b32 + the accumulating v_bcnt_u32_b32), so the kernel is organised to issue nothing
// else in the inner loop:
//   * "P" operand rows live one-per-lane: a wave owns 64 * kTP rows of P and reads their packed
//     words from an LDS tile (padded so that 8-byte reads are bank-conflict free).
//   * "Q" operand rows are wave-uniform: each wave owns kTQ rows of Q and fetches their words
//     with scalar loads into SGPRs, which v_xor_b32 takes as a free operand.  No VGPR, LDS or
//     vector-memory traffic is spent on Q bits.  The scalar loads are written as inline asm (row
//     offset in the instruction's SGPR-offset field, no per-load address arithmetic) and are
//     waited for explicitly; check_isa.py verifies on the compiled ISA that nothing touches their
//     destination registers before that wait.
//   * each lane keeps kTP x kTQ integer accumulators and as many fp32 results.
//   * the popcount accumulator of a segment is seeded with -G/2 (first v_bcnt of the segment takes
//     the seed instead of the old value, so no reset instruction exists); then d = -2 * acc and the
//     factor -2 is folded into the P scale.  Epilogue per accumulator per segment: cvt, mul, fma.
//   * K is walked in chunks of kCK words; the next chunk's P words and both operands' scales are
//     fetched from global memory while the current chunk is being reduced, then parked in the
//     other LDS buffer (one barrier per chunk).  A workgroup is 4 waves (tile 128 x 64) and three or
//     four workgroups share a CU, so one group's barrier and LDS refill overlap the others' arithmetic.
// Either of A / B can be P or Q: the host picks the role by output strides.
#include "kernels.h"
#include "tile_map.h"
#include "wave_ops.h"

namespace hbmm {
namespace {

constexpr int kTQMax = 16;             // Q rows per wave: 16, or fewer when that balances the grid (see the launcher)
constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;  // 256
constexpr int kSlotsQ = kTQMax * kWaves;   // Q scale slots per segment in LDS (wave w owns slots 16 w .. 16 w + 15)
constexpr int kCK = 16;                // 32-bit words of K per chunk (512 bits)
constexpr int kStep = 2;               // words per inner step (one 8-byte LDS read, one s_load_dwordx2)
constexpr int kBitsStride = kCK + 2;   // LDS row stride in words: 2 * odd => conflict-free b64 reads

typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// popcount(x) + acc in one instruction.  Written as asm so that the optimiser cannot re-associate
// chains of these into separate popcounts plus three-operand adds.
__device__ __forceinline__ int bcnt_acc(uint32_t x, int acc)
{
    int d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
    return d;
}
__device__ __forceinline__ int bcnt_seed(uint32_t x, int seed)
{
    int d;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "s"(seed));
    return d;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// FUSED: the P operand is given as fp32 (a.p_src) and is binarised inside the kernel, chunk by chunk,
// straight into the LDS tile -- the packed form of P never exists in memory.
//
// TP = P rows per lane.  2 (a workgroup owns 128 rows of P; 128 to 166 registers per lane, so three or
// four workgroups share a compute unit and cover each other's waits) is the form for grids that fill
// the chip: it is 6 to 15 % faster than 4 rows per lane with two workgroups per compute unit, and
// 1 row per lane is slower again (the scalar loads of Q are then shared by too little arithmetic).
// 1 (64 rows) is used for small problems, which then spread over twice as many workgroups; 4 (256
// rows) for a K of at most two chunks on a large grid.  The fused form uses 2 and 1 the same way.
//
// TQ = Q rows per wave (a workgroup owns 4 TQ rows of Q).  16 unless the launcher finds that a smaller
// tile spreads the work more evenly over the compute units.
template <int G, bool INTEGER, bool FUSED, int TP, int TQ>
__global__ __launch_bounds__(kThreads, TP == 2 ? (G >= 128 && !FUSED ? 4 : 3) : 2) void popcount_gemm_kernel(const PopcountGemmArgs a)
{
    static_assert(TQ == 1 || TQ == 2 || TQ == 4 || (TQ >= 12 && TQ <= 14) || TQ == kTQMax,
                  "wait_q() below is written out for 1, 2, 4, 12, 13, 14 and 16 rows");
    constexpr int kTP = TP;
    constexpr int kTQ = TQ;
    constexpr int kTileQ = kTQ * kWaves;                        // Q rows per workgroup
    constexpr int kTileP = 64 * TP;                             // P rows per workgroup
    constexpr int kRowsPerWave = kTileP / kWaves;                // rows of P a wave binarises in the fused form
    constexpr int kWordsPerGran = G / 32;                       // 1, 2, 4, 8
    constexpr int kGranPerChunk = kCK / kWordsPerGran;          // 16, 8, 4, 2
    constexpr int kSteps = kCK / kStep;                         // 8
    // Scaled mode: a segment's accumulator starts at the bit pattern of 2^23 and v_bcnt adds the
    // Hamming count to it as an integer, so the register always holds the *float* 2^23 + hamming
    // (exact: counts are far below 2^23).  The epilogue gets hamming - G/2 with one fp32 subtraction,
    // which issues at twice the rate of the integer-to-float conversion it replaces.
    constexpr int kSeed = INTEGER ? 0 : 0x4b000000;
    constexpr float kSeedValue = 8388608.0f + (float)(G / 2);

    __shared__ __attribute__((aligned(16))) uint32_t s_bits[2][kTileP * kBitsStride];
    constexpr int kScaleStrideP = kGranPerChunk + 1;   // odd => conflict-free b32 reads
    __shared__ __attribute__((aligned(16))) float s_ps[INTEGER ? 1 : 2][INTEGER ? 1 : kTileP * kScaleStrideP];
    __shared__ __attribute__((aligned(16))) float s_qs[INTEGER ? 1 : 2][INTEGER ? 1 : kGranPerChunk * kSlotsQ];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroup -> tile: super-tiles of 128 tiles, dealt evenly to the 8 XCDs (tile_map.h).
    int tile_p, tile_q;
    if (!popcount_map_tile(blockIdx.x, a.tiles_p, a.tiles_q, a.sup_p, tile_p, tile_q)) return;
    const int p0 = tile_p * kTileP;
    const int q0_wg = tile_q * kTileQ;
    const int q0 = q0_wg + wave * kTQ;

    const int nchunks = (a.kwords + kCK - 1) / kCK;
    // scale entries per chunk for each operand: 512 / beta = kGranPerChunk >> shift
    const int nsp = INTEGER ? 0 : (kGranPerChunk >> a.shift_p);
    const int nsq = INTEGER ? 0 : (kGranPerChunk >> a.shift_q);
    const int nblk_p = INTEGER ? 0 : a.nblk_p;
    const int nblk_q = INTEGER ? 0 : a.nblk_q;

    // ---- staging registers for the next chunk
    constexpr int kBitPieces = kTileP * (kCK / 4) / kThreads;             // 2 x 16 bytes per thread
    constexpr int kPsPerThread = (kTileP * kGranPerChunk + kThreads - 1) / kThreads;   // <= 8
    constexpr int kQsPerThread = (kSlotsQ * kGranPerChunk + kThreads - 1) / kThreads;  // <= 4
    uint4 st_bits[kBitPieces];
    float st_ps[INTEGER ? 1 : kPsPerThread];
    float st_qs[INTEGER ? 1 : kQsPerThread];

    uint32_t st_qline = 0;
    auto fetch = [&](int chunk) {
        // Touch the 64-byte line of this wave's Q rows that the scalar loads of `chunk` will read,
        // one chunk ahead, through the vector path (its counter is separate from the scalar one), so
        // that those scalar loads find the line in L2.
        if (lane < kTQ) {
            const int row = min(q0 + lane, a.Q - 1);
            const int w = min(chunk * kCK, a.kwords - 4);
            st_qline = a.q_bits[(int64_t)row * a.ldw_q + w];
        }
        if constexpr (!FUSED) {
#pragma unroll
            for (int r = 0; r < kBitPieces; ++r) {
                const int id = tid + r * kThreads;
                const int row = p0 + id / (kCK / 4);
                const int w = chunk * kCK + (id % (kCK / 4)) * 4;
                st_bits[r] = make_uint4(0, 0, 0, 0);
                if (row < a.P && w < a.kwords)
                    st_bits[r] = *reinterpret_cast<const uint4 *>(a.p_bits + (int64_t)row * a.ldw_p + w);
            }
        }
        if constexpr (!INTEGER) {
            if constexpr (!FUSED) {
#pragma unroll
                for (int r = 0; r < kPsPerThread; ++r) {
                    const int id = tid + r * kThreads;
                    const int row = p0 + id / kGranPerChunk;
                    const int e = id % kGranPerChunk;
                    const int blk = chunk * nsp + e;
                    st_ps[r] = 0.f;
                    if (id < kTileP * kGranPerChunk && e < nsp && row < a.P && blk < nblk_p)
                        st_ps[r] = a.p_scales[(int64_t)row * a.lds_p + blk];
                }
            }
#pragma unroll
            for (int r = 0; r < kQsPerThread; ++r) {
                const int id = tid + r * kThreads;
                const int slot = id / kGranPerChunk;          // wave (slot / 16) and its row (slot % 16)
                const int row = q0_wg + (slot >> 4) * kTQ + (slot & 15);
                const int e = id % kGranPerChunk;
                const int blk = chunk * nsq + e;
                st_qs[r] = 0.f;
                if (id < kSlotsQ * kGranPerChunk && (slot & 15) < kTQ && e < nsq && row < a.Q && blk < nblk_q)
                    st_qs[r] = a.q_scales[(int64_t)row * a.lds_q + blk];
            }
        }
    };
    auto park = [&](int buf) {
        asm volatile("" ::"v"(st_qline));   // keeps the touch load alive; its value is not used
        if constexpr (!FUSED) {
#pragma unroll
            for (int r = 0; r < kBitPieces; ++r) {
                const int id = tid + r * kThreads;
                const int row = id / (kCK / 4);
                const int w = (id % (kCK / 4)) * 4;
                uint32_t *dst = &s_bits[buf][row * kBitsStride + w];
                // rows start at an 8-byte boundary only (stride 18 words): two 8-byte stores
                *reinterpret_cast<uint2 *>(dst) = make_uint2(st_bits[r].x, st_bits[r].y);
                *reinterpret_cast<uint2 *>(dst + 2) = make_uint2(st_bits[r].z, st_bits[r].w);
            }
        }
        if constexpr (!INTEGER) {
            if constexpr (!FUSED) {
#pragma unroll
                for (int r = 0; r < kPsPerThread; ++r) {
                    const int id = tid + r * kThreads;
                    if (id < kTileP * kGranPerChunk)
                        s_ps[buf][(id / kGranPerChunk) * kScaleStrideP + id % kGranPerChunk] = st_ps[r];
                }
            }
#pragma unroll
            for (int r = 0; r < kQsPerThread; ++r) {
                const int id = tid + r * kThreads;
                if (id < kSlotsQ * kGranPerChunk)
                    s_qs[buf][(id % kGranPerChunk) * kSlotsQ + id / kGranPerChunk] = st_qs[r];
            }
        }
    };

    // ---- FUSED: binarise chunk `chunk` of this workgroup's P rows from fp32 into LDS buffer `buf`.
    // A wave owns kRowsPerWave rows; per row the chunk is 512 elements = two 16-byte loads per lane (lane l holds
    // elements 4l .. 4l+3 of each half).  Signs, words and scales are produced exactly as in the
    // stand-alone pack kernel (same nibble merge, same pairwise order of the |x| sums), so the scales
    // are bit-identical to packing first.
    // Rows are handled in batches of kPackRows with two register sets: while one batch is turned into
    // words the loads of the next are in flight, and the first batch of the next chunk is requested
    // before the popcount phase of this one, so that the memory pipe is never idle.
    constexpr int kPackRows = 4;
    constexpr int kPackBatches = kRowsPerWave / kPackRows;
    static_assert(kPackBatches % 2 == 0, "batches are worked in pairs");
    f32x4 pv[FUSED ? 2 : 1][FUSED ? kPackRows : 1][2];
    auto pack_issue = [&](int chunk, int b, f32x4 (&v)[FUSED ? kPackRows : 1][2]) {
        if constexpr (FUSED) {
            // past the end of K or P the addresses are clamped; such values are masked when used
            const int k_lane = chunk * (kCK * 32) + 4 * lane;
#pragma unroll
            for (int j = 0; j < kPackRows; ++j) {
                const int row = p0 + wave * kRowsPerWave + b * kPackRows + j;
                const float *src = a.p_src + (int64_t)min(row, a.P - 1) * a.ld_p_src;
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    v[j][h] = __builtin_nontemporal_load(
                        reinterpret_cast<const f32x4 *>(src + min(k_lane + h * 256, a.K - 4)));
            }
        }
    };
    // The batch is worked through phase by phase (all words, then each level of the scale sums, then
    // the LDS stores) so that the eight row-halves give eight independent dependency chains per phase
    // and every branch is taken once per batch.  Lanes past K or rows past P work on clamped loads:
    // K is a multiple of beta, so no word or segment mixes live and dead elements, and dead words and
    // scales are never read.  A half that lies wholly past K (last chunk only) is skipped.
    auto pack_words = [&](int chunk, int b, const f32x4 (&v)[FUSED ? kPackRows : 1][2], int buf) {
        if constexpr (FUSED) {
            const int seg_lanes = a.beta_p >> 2;               // lanes per P segment: 8 .. 64
            const float inv_beta = 1.0f / (float)a.beta_p;
            const int halves = (chunk * (kCK * 32) + 256 < a.K) ? 2 : 1;
            uint32_t word[kPackRows][2];
            float sum[kPackRows][2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (h < halves) {
#pragma unroll
                    for (int j = 0; j < kPackRows; ++j) {
                        const f32x4 x = v[j][h];
                        const uint32_t nib = (x.x >= 0.f ? 1u : 0u) | (x.y >= 0.f ? 2u : 0u) |
                                             (x.z >= 0.f ? 4u : 0u) | (x.w >= 0.f ? 8u : 0u);
                        word[j][h] = pack_word_from_nibbles(nib, lane);
                        if constexpr (!INTEGER)
                            sum[j][h] = segment_sum<8>((fabsf(x.x) + fabsf(x.y)) + (fabsf(x.z) + fabsf(x.w)));
                    }
                }
            }
            if constexpr (!INTEGER) {
                if (seg_lanes >= 16) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < kPackRows; ++j)
                            if (h < halves) sum[j][h] += dpp_f32<kDppRowMirror>(sum[j][h]);
                }
                if (seg_lanes >= 32) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < kPackRows; ++j)
                            if (h < halves) sum[j][h] += __shfl_xor(sum[j][h], 16);
                }
                if (seg_lanes >= 64) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < kPackRows; ++j)
                            if (h < halves) sum[j][h] += __shfl_xor(sum[j][h], 32);
                }
            }
            const int row_l = wave * kRowsPerWave + b * kPackRows;
            if ((lane & 7) == 0) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int j = 0; j < kPackRows; ++j)
                        if (h < halves) s_bits[buf][(row_l + j) * kBitsStride + h * 8 + (lane >> 3)] = word[j][h];
            }
            if constexpr (!INTEGER) {
                if ((lane & (seg_lanes - 1)) == 0) {
                    const int e = (4 * lane) / a.beta_p;
                    const int e_half = 256 / a.beta_p;
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int j = 0; j < kPackRows; ++j)
                            if (h < halves)
                                s_ps[buf][(row_l + j) * kScaleStrideP + h * e_half + e] = sum[j][h] * inv_beta;
                }
            }
        }
    };
    // Expects batch 0 of `chunk` to have been requested into pv[0]; leaves batch 0 of chunk + 1 there.
    auto pack_chunk = [&](int chunk, int buf) {
        if constexpr (FUSED) {
            if (chunk >= nchunks) return;
#pragma unroll 1
            for (int b = 0; b < kPackBatches; b += 2) {
                pack_issue(chunk, b + 1, pv[1]);
                pack_words(chunk, b, pv[0], buf);
                const bool more = b + 2 < kPackBatches;
                pack_issue(more ? chunk : chunk + 1, more ? b + 2 : 0, pv[0]);
                pack_words(chunk, b + 1, pv[1], buf);
            }
        }
    };

    // ---- accumulators
    int acc[kTP][kTQ];
    float res[INTEGER ? 1 : kTP][INTEGER ? 1 : kTQ];
#pragma unroll
    for (int i = 0; i < kTP; ++i)
#pragma unroll
        for (int q = 0; q < kTQ; ++q) {
            acc[i][q] = kSeed;
            if (!INTEGER) res[i][q] = 0.f;
        }

    // scalar-side row offsets in bytes (rows past Q re-read row Q-1; their results are never stored)
    typedef const char __attribute__((address_space(4))) *const_byte_ptr;
    const const_byte_ptr qbase = (const_byte_ptr)a.q_bits;
    uint32_t qoff[kTQ];
#pragma unroll
    for (int q = 0; q < kTQ; ++q) qoff[q] = (uint32_t)(min(q0 + q, a.Q - 1) * a.ldw_q) * 4u;

    pack_issue(0, 0, pv[0]);
    fetch(0);
    park(0);
    pack_chunk(0, 0);
    __syncthreads();

    // Scales of segment g_local of the chunk in `buf`: sp = -2 * sP (folds d = -2 * acc), sq = sQ.
    auto load_scales = [&](float (&sp)[kTP], float (&sq)[kTQ], int buf, int g_local) {
#pragma unroll
        for (int i = 0; i < kTP; ++i)
            sp[i] = s_ps[buf][(lane + 64 * i) * kScaleStrideP + (g_local >> a.shift_p)];
        const float4 *sq4 =
            reinterpret_cast<const float4 *>(&s_qs[buf][(g_local >> a.shift_q) * kSlotsQ + wave * kTQMax]);
#pragma unroll
        for (int v = 0; v < (kTQ + 3) / 4; ++v) {
            const float4 t = sq4[v];
            const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * v + j < kTQ) sq[4 * v + j] = tv[j];
        }
    };
    // Epilogue of one segment: res += (hamming - G/2) * (-2 sP * sQ)  (-2 (hamming - G/2) = d).  The
    // scale product is formed first so that the result does not depend on which operand is P.
    auto epilogue = [&](const float (&sp)[kTP], const float (&sq)[kTQ]) {
#pragma unroll
        for (int i = 0; i < kTP; ++i) {
            const float sp2 = -2.0f * sp[i];
#pragma unroll
            for (int q = 0; q < kTQ; ++q)
                res[i][q] = __builtin_fmaf(__builtin_bit_cast(float, acc[i][q]) - kSeedValue, sp2 * sq[q], res[i][q]);
        }
        // Pin the results here: without a use at this point the optimiser sinks the whole epilogue
        // to the end of the chunk and keeps every segment's accumulators alive until then.
#pragma unroll
        for (int i = 0; i < kTP; ++i)
#pragma unroll
            for (int q = 0; q < kTQ; ++q) asm volatile("" : "+v"(res[i][q]));
        __builtin_amdgcn_sched_barrier(0);
    };
    // The shorter last segment of a K that G does not divide: `bits` of it exist, so its inner product is
    // bits - 2 * hamming (the pad bits of both operands are 0 and xor to 0).  Ragged tail loop only.
    auto epilogue_tail = [&](const float (&sp)[kTP], const float (&sq)[kTQ], int bits) {
        // (the hamming count first, exactly; half of an odd `bits` is not a float next to 2^23)
        const float half = 0.5f * (float)bits;
#pragma unroll
        for (int i = 0; i < kTP; ++i) {
            const float sp2 = -2.0f * sp[i];
#pragma unroll
            for (int q = 0; q < kTQ; ++q)
                res[i][q] = __builtin_fmaf((__builtin_bit_cast(float, acc[i][q]) - 8388608.0f) - half, sp2 * sq[q],
                                           res[i][q]);
        }
    };
    // Scalar loads of Q words, written as asm so that the row offset can ride in the instruction's
    // SGPR-offset field (no address arithmetic per load).  The compiler does not count these loads,
    // so wait_q() must run before their results are read: it waits for every outstanding scalar /
    // LDS access and ties the 16 results to itself so that no use can be scheduled above it.
    auto load_q = [&](u32x2 (&qw)[kTQ], int step_index, int wbase) {
        const uint64_t base = (uint64_t)qbase + (uint64_t)(wbase + step_index * kStep) * 4u;
#pragma unroll
        for (int q = 0; q < kTQ; ++q)
            asm volatile("s_load_dwordx2 %0, %1, %2" : "=s"(qw[q]) : "s"(base), "s"(qoff[q]));
    };
    auto wait_q = [&](u32x2 (&qw)[kTQ]) {
#define HBMM_QW2 "+s"(qw[0]), "+s"(qw[1])
#define HBMM_QW4 HBMM_QW2, "+s"(qw[2]), "+s"(qw[3])
#define HBMM_QW12 HBMM_QW4, "+s"(qw[4]), "+s"(qw[5]), "+s"(qw[6]), "+s"(qw[7]), "+s"(qw[8]), "+s"(qw[9]), "+s"(qw[10]), "+s"(qw[11])
        if constexpr (kTQ == 16)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW12, "+s"(qw[12]), "+s"(qw[13]), "+s"(qw[14]), "+s"(qw[15]));
        else if constexpr (kTQ == 14)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW12, "+s"(qw[12]), "+s"(qw[13]));
        else if constexpr (kTQ == 13)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW12, "+s"(qw[12]));
        else if constexpr (kTQ == 12)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW12);
        else if constexpr (kTQ == 4)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW4);
        else if constexpr (kTQ == 2)
            asm volatile("s_waitcnt lgkmcnt(0)" : HBMM_QW2);
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(qw[0]));
#undef HBMM_QW12
#undef HBMM_QW4
#undef HBMM_QW2
    };
    auto load_p = [&](u32x2 (&pw)[kTP], int buf, int s) {
        const uint32_t *lbits = &s_bits[buf][lane * kBitsStride + s * kStep];
#pragma unroll
        for (int i = 0; i < kTP; ++i) pw[i] = *reinterpret_cast<const u32x2 *>(lbits + i * 64 * kBitsStride);
    };
    // One word of one half of the Q rows: 32 x (v_xor_b32 + v_bcnt_u32_b32).
    auto reduce_half = [&](const uint32_t (&pwv)[kTP], const uint32_t (&qwv)[kTQ], int half, bool first) {
#pragma unroll
        for (int q = half ? kTQ / 2 : 0; q < (half ? kTQ : kTQ / 2); ++q)
#pragma unroll
            for (int i = 0; i < kTP; ++i)
                acc[i][q] = first ? bcnt_seed(pwv[i] ^ qwv[q], kSeed) : bcnt_acc(pwv[i] ^ qwv[q], acc[i][q]);
    };

    // Chunks whose 16 words all lie inside K: branch-free and fully unrolled.  Per step the first
    // half of the Q rows is reduced (its first instruction absorbs the wait for this step's
    // operands), then the next step's operands are requested, then the second half is reduced
    // while those requests are in flight.
    const int nfull = INTEGER ? a.kwords / kCK : (a.ngran * kWordsPerGran) / kCK;
    int chunk = 0;
    for (; chunk < nfull; ++chunk) {
        const int buf = chunk & 1;
        fetch(chunk + 1);   // past the last chunk every guard fails and zeros are staged
        const int wbase = chunk * kCK;

        u32x2 pw[2][kTP];
        u32x2 qw[2][kTQ];
        float sp[kTP], sq[kTQ];
        load_p(pw[0], buf, 0);
        load_q(qw[0], 0, wbase);
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const int cur = s & 1;
            const bool first0 = !INTEGER && ((s * kStep) % kWordsPerGran == 0);
            const bool first1 = !INTEGER && ((s * kStep + 1) % kWordsPerGran == 0);
            const bool last0 = !INTEGER && ((s * kStep + 1) % kWordsPerGran == 0);
            const bool last1 = !INTEGER && ((s * kStep + 2) % kWordsPerGran == 0);
            uint32_t px[kTP], py[kTP], qx[kTQ], qy[kTQ];
            wait_q(qw[cur]);
#pragma unroll
            for (int i = 0; i < kTP; ++i) { px[i] = pw[cur][i].x; py[i] = pw[cur][i].y; }
#pragma unroll
            for (int q = 0; q < kTQ; ++q) {
                qx[q] = qw[cur][q].x;
                qy[q] = qw[cur][q].y;
            }

            if (last0) {
                // one-word segments: both words end a segment; no room to hide the scale reads
                reduce_half(px, qx, 0, first0);
                reduce_half(px, qx, 1, first0);
                load_scales(sp, sq, buf, (s * kStep) / kWordsPerGran);
                epilogue(sp, sq);
                reduce_half(py, qy, 0, first1);
                __builtin_amdgcn_sched_barrier(0);
                if (s + 1 < kSteps) {
                    load_p(pw[cur ^ 1], buf, s + 1);
                    load_q(qw[cur ^ 1], s + 1, wbase);
                }
                load_scales(sp, sq, buf, (s * kStep + 1) / kWordsPerGran);
                __builtin_amdgcn_sched_barrier(0);
                reduce_half(py, qy, 1, first1);
                epilogue(sp, sq);
            } else {
                reduce_half(px, qx, 0, first0);
                reduce_half(py, qy, 0, first1);
                __builtin_amdgcn_sched_barrier(0);
                if (s + 1 < kSteps) {
                    load_p(pw[cur ^ 1], buf, s + 1);
                    load_q(qw[cur ^ 1], s + 1, wbase);
                }
                if (last1) load_scales(sp, sq, buf, (s * kStep + 1) / kWordsPerGran);
                __builtin_amdgcn_sched_barrier(0);
                reduce_half(px, qx, 1, first0);
                reduce_half(py, qy, 1, first1);
                if (last1) epilogue(sp, sq);
            }
        }
        park(buf ^ 1);
        pack_chunk(chunk + 1, buf ^ 1);
        __syncthreads();
    }
    // Ragged last chunk (at most one): word-at-a-time loop with explicit accumulator resets.
    if (!INTEGER && chunk < nchunks) {
#pragma unroll
        for (int i = 0; i < kTP; ++i)
#pragma unroll
            for (int q = 0; q < kTQ; ++q) acc[i][q] = kSeed;
    }
    for (; chunk < nchunks; ++chunk) {
        const int buf = chunk & 1;
        const int wbase = chunk * kCK;
        for (int w = 0; w < kCK && wbase + w < a.kwords; ++w) {
            uint32_t pw1[kTP];
#pragma unroll
            for (int i = 0; i < kTP; ++i) pw1[i] = s_bits[buf][(lane + 64 * i) * kBitsStride + w];
#pragma unroll
            for (int q = 0; q < kTQ; ++q) {
                const uint32_t qw1 = *(const_u32_ptr)(qbase + (uint64_t)qoff[q] + (int64_t)(wbase + w) * 4);
#pragma unroll
                for (int i = 0; i < kTP; ++i) acc[i][q] += __builtin_popcount(pw1[i] ^ qw1);
            }
            if (!INTEGER && a.tail_bits > 0 && wbase + w + 1 == a.kw_used) {
                // the last word that holds elements: the segment that ends here is shorter than G
                float sp[kTP], sq[kTQ];
                load_scales(sp, sq, buf, w / kWordsPerGran);
                epilogue_tail(sp, sq, a.tail_bits);
            }
            if (!INTEGER && (w + 1) % kWordsPerGran == 0) {
                const int g_local = w / kWordsPerGran;
                if (chunk * kGranPerChunk + g_local < a.ngran) {
                    float sp[kTP], sq[kTQ];
                    load_scales(sp, sq, buf, g_local);
                    epilogue(sp, sq);
                }
#pragma unroll
                for (int i = 0; i < kTP; ++i)
#pragma unroll
                    for (int q = 0; q < kTQ; ++q) acc[i][q] = kSeed;
            }
        }
    }

    // ---- store.  When Q runs along the rows of the output (ld_out_q == 1: P is the M side), a lane's 16
    // results of one P row are contiguous: four 16-byte stores instead of sixteen 4-byte ones.
    const bool row_vectors = kTQ % 4 == 0 && a.ld_out_q == 1 && (a.ld_out_p & 3) == 0 && q0 + kTQ <= a.Q;
#pragma unroll
    for (int i = 0; i < kTP; ++i) {
        const int p = p0 + lane + 64 * i;
        if (p >= a.P) continue;
        uint32_t v[kTQ];
#pragma unroll
        for (int q = 0; q < kTQ; ++q)
            v[q] = INTEGER ? (uint32_t)(a.K - 2 * acc[i][q]) : __builtin_bit_cast(uint32_t, res[INTEGER ? 0 : i][INTEGER ? 0 : q]);
        uint32_t *dst = reinterpret_cast<uint32_t *>(a.out);
        if (row_vectors) {
            uint4 *d4 = reinterpret_cast<uint4 *>(dst + (int64_t)p * a.ld_out_p + q0);
#pragma unroll
            for (int c = 0; c < kTQ / 4; ++c) d4[c] = make_uint4(v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]);
        } else {
#pragma unroll
            for (int q = 0; q < kTQ; ++q) {
                const int qq = q0 + q;
                if (qq < a.Q) dst[(int64_t)p * a.ld_out_p + (int64_t)qq * a.ld_out_q] = v[q];
            }
        }
    }
}

template <int G, bool INTEGER, bool FUSED = false, int TP = 4, int TQ = kTQMax>
hipError_t launch(const PopcountGemmArgs &a, hipStream_t s)
{
    int64_t nblocks = (int64_t)a.tiles_p * a.tiles_q;
    if (nblocks <= 0) return hipSuccess;
    if (nblocks > 0x7fffff00LL) return hipErrorInvalidConfiguration;
    nblocks = popcount_map_blocks(a.tiles_p, a.tiles_q, a.sup_p);
    popcount_gemm_kernel<G, INTEGER, FUSED, TP, TQ><<<dim3((unsigned)nblocks), dim3(kThreads), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_popcount_gemm(const PopcountGemmArgs &args, int G, int integer, hipStream_t s)
{
    PopcountGemmArgs a = args;
    constexpr int kTileQ = kTQMax * kWaves;
    a.tiles_q = (a.Q + kTileQ - 1) / kTileQ;
    // 128 rows of P per workgroup (three workgroups share a compute unit), or 64 when that grid would
    // leave compute units without a workgroup (small problems are bound by the length of one
    // workgroup's work).
    const bool fused = a.p_src != nullptr;
    const bool narrow = (int64_t)((a.P + 127) / 128) * a.tiles_q < 256;
    // (a K of at most two chunks on a grid that fills the chip either way: 256 rows, i.e. half as many
    // workgroup starts and ends, measured 10 % faster on 200704 x 576 x 64)
    // (not for 32-bit segments: four rows per lane do not fit the registers there)
    const bool wide = !fused && !narrow && !integer && G != 32 && a.kwords <= 2 * kCK &&
                      (int64_t)((a.P + 255) / 256) * a.tiles_q >= 512;
    const int tile_p = wide ? 256 : narrow ? 64 : 128;
    a.tiles_p = (a.P + tile_p - 1) / tile_p;
    // super-tile shape: sup_p x (128 / sup_p) tiles, 16 x 8 when P has that many tiles (2048 rows of P and
    // 512 of Q: 2.5 MB of packed bits at K = 8192, inside one XCD's 4 MB L2); measured against 4 x 16,
    // 8 x 8, 32 x 4 and super-tiles of 64, 256 and 512 tiles
    a.sup_p = a.tiles_p >= 16 ? 16 : a.tiles_p >= 4 ? 4 : (a.tiles_p >= 2 ? 2 : 1);
    if ((int64_t)a.tiles_p * a.tiles_q <= 2 * kMapXcds * kMapSuperTiles) a.sup_p = 0;   // at most two rounds: plain map
    if (integer) return narrow ? launch<64, true, false, 1>(a, s) : launch<64, true, false, 2>(a, s);
    if (fused) {
        switch (G) {
        case 32: return narrow ? launch<32, false, true, 1>(a, s) : launch<32, false, true, 2>(a, s);
        case 64: return narrow ? launch<64, false, true, 1>(a, s) : launch<64, false, true, 2>(a, s);
        case 128: return narrow ? launch<128, false, true, 1>(a, s) : launch<128, false, true, 2>(a, s);
        case 256: return narrow ? launch<256, false, true, 1>(a, s) : launch<256, false, true, 2>(a, s);
        }
        return hipErrorInvalidValue;
    }
    if (narrow) {
        // A grid this small is bound by the length of one workgroup's work, not by throughput: take the
        // fewest rows of Q per wave (1, 2, 4 or 16) that still give every workgroup a compute unit of its
        // own.  Kernel durations, 16 rows -> chosen: 64 x 64 x 512 at 32-bit segments 7.5 -> 4.8 us (1 row,
        // 16 workgroups); 3136 x 64 x 576 at 64 bits 8.4 -> 5.5 us (4 rows, 196 workgroups); 70 x 50 x 992
        // 15.1 -> 6.2 us; 1000 x 100 x 2048 at 256 bits 12.6 -> 6.0 us.  What remains is launch and latency.
        int tqn = kTQMax;
        for (int t : {1, 2, 4})
            if ((int64_t)a.tiles_p * ((a.Q + kWaves * t - 1) / (kWaves * t)) <= 256) {
                tqn = t;
                break;
            }
        if (tqn != kTQMax) a.tiles_q = (a.Q + kWaves * tqn - 1) / (kWaves * tqn);
#define HBMM_POPCOUNT_NARROW(GV)                                              \
    switch (tqn) {                                                            \
    case 1: return launch<GV, false, false, 1, 1>(a, s);                      \
    case 2: return launch<GV, false, false, 1, 2>(a, s);                      \
    case 4: return launch<GV, false, false, 1, 4>(a, s);                      \
    default: return launch<GV, false, false, 1>(a, s);                        \
    }
        switch (G) {
        case 32: HBMM_POPCOUNT_NARROW(32)
        case 64: HBMM_POPCOUNT_NARROW(64)
        case 128: HBMM_POPCOUNT_NARROW(128)
        case 256: HBMM_POPCOUNT_NARROW(256)
        }
#undef HBMM_POPCOUNT_NARROW
        return hipErrorInvalidValue;
    }
    if (wide) {
        switch (G) {
        case 64: return launch<64, false, false, 4>(a, s);
        case 128: return launch<128, false, false, 4>(a, s);
        case 256: return launch<256, false, false, 4>(a, s);
        }
        return hipErrorInvalidValue;
    }
    // Rows of Q per wave.  All workgroups of a launch are about equally long and a compute unit works on
    // its share of them side by side, so the launch lasts as long as the unit with the most workgroups:
    // ceil(tiles / 256) workgroups of 4 tq rows.  12544 x 512 with 64-row tiles is 784 tiles -- 3.06 per
    // unit, so the launch takes as long as 4 per unit would (measured: 16384 rows take the same 92 us as
    // 12544, 12288 rows take 73) -- while 52-row tiles give 968, still 4 per unit, each 13/16 as long.
    // A smaller tile is taken only for a modelled gain of 8 % or more: its fixed costs weigh more (so 15
    // rows are never chosen).  Measured, 16 / 14 / 13 / 12 rows per wave: 12544 x 512 x 4608 at 128-bit
    // segments 95 / 84 / 81 / 88 us, 50176 x 128 x 1152 at 64-bit segments 38 / 33 / 29 / 33 us,
    // 9000 x 512 x 2048 at 256-bit segments 33 / 30 / 28 / 27 us; the model picks 13, 13 and 12.
    int tq = kTQMax;
    {
        auto rounds = [&](int t) {
            const int64_t tiles = (int64_t)a.tiles_p * ((a.Q + kWaves * t - 1) / (kWaves * t));
            return (double)((tiles + 255) / 256) * t;
        };
        double best = rounds(kTQMax) * 0.92;
        for (int t = 14; t >= 12; --t)
            if (rounds(t) < best) {
                best = rounds(t);
                tq = t;
            }
    }
    if (tq != kTQMax) {
        a.tiles_q = (a.Q + kWaves * tq - 1) / (kWaves * tq);
        if ((int64_t)a.tiles_p * a.tiles_q <= 2 * kMapXcds * kMapSuperTiles) a.sup_p = 0;
    }
#define HBMM_POPCOUNT_TQ(GV)                                                  \
    switch (tq) {                                                             \
    case 12: return launch<GV, false, false, 2, 12>(a, s);                    \
    case 13: return launch<GV, false, false, 2, 13>(a, s);                    \
    case 14: return launch<GV, false, false, 2, 14>(a, s);                    \
    default: return launch<GV, false, false, 2>(a, s);                        \
    }
    switch (G) {
    case 32: HBMM_POPCOUNT_TQ(32)
    case 64: HBMM_POPCOUNT_TQ(64)
    case 128: HBMM_POPCOUNT_TQ(128)
    case 256: HBMM_POPCOUNT_TQ(256)
    }
#undef HBMM_POPCOUNT_TQ
    return hipErrorInvalidValue;
}

}  // namespace hbmm
