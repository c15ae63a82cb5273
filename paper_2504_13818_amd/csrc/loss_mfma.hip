// Matrix-core kernels for the GRPO-PODS token loss with bf16 inputs (gfx950).
//
// The packed token rows are processed in blocks of nb rows (32768 by default).  Per block, three
// contractions run as one workgroup per 256x256 output tile with fp32 accumulators: the logits with
// v_mfma_f32_32x32x16_bf16 on transposed copies of the bf16 inputs, the two gradient contractions with
// v_mfma_f32_32x32x16_f16 on fp16 working copies (exact while the scaled value stays in fp16's normal
// range):
//
//   forward    z[v][t]  = sum_k Wt[k][v]  Ht[k][t]      -> per token and vocabulary tile: an integer E with
//                                                          2^(E+2) > exp(max z), sum exp(z) 2^-E, z_y, and the
//                                                          numerators 2^14 exp(z) 2^-E as fp16
//   normalise  q[t][v]  = numerator * 2^(E - Eref_t)    -> q = 2^14 softmax / c_t (0 at v = y), in place, exact;
//                                                          only where E differs from Eref_t = max E of the token
//   d_hidden   dH[k][t] = sum_v W16[v][k] q[t][v]       -> times -g_t, over the whole vocabulary
//   d_w_lm     dW[k][v] = sum_t H16[t][k] q[t][v]       -> accumulated over the token blocks
//
// The softmax numerators of ONE token block, q[nb][V], are the only [tokens, vocabulary]-shaped array that
// ever exists (10 GB of the 90 GB the full logits would take at the Qwen2.5-3B-shaped sizes): keeping them
// from the forward pass, under a power-of-two offset per (token, vocabulary tile), spares the backward pass a
// second logits contraction (2 N d V of the 8 N d V floating-point operations a recomputing backward pass
// executes).  After a block's first forward launch (the first 8192 vocabulary columns) every token fixes the
// exponent its later tiles use: four above the larger of the first launch's exponents and that of the generated
// token's own logit, which a policy that sampled the token has made large.  A tile takes the agreed exponent
// unless its own lies two or more above it, so for nearly every token all later tiles share one offset and the
// normalising pass has only the first launch's tiles (and such rare tokens) to touch; the remaining per-token
// factor c_t = 2^Eref exp(-lse) rides on the token's weight g_t.
//
// An operand whose contraction index is its row index in memory (all of them except q in
// d_hidden) is staged in LDS as it lies in memory and read with the transposing LDS load, so q is
// stored once (token-major) and no transposed copy of q or of the gradient operands exists; the
// logits read blocked transposed copies Wt, Ht made once per call.
//
// The per-logit gradient is dz = -g_t q / 2^14 for v != y.  q is kept in fp16 (11-bit significand)
// rather than bf16 (8-bit) so that a logit with a large probability does not carry a 2^-8 error
// into its token's gradient.  The token weight g_t, which spans many binades, never enters q:
// d_hidden applies it per output row, and d_w_lm folds it into H16 = fp16(s g_t h_t) with one
// power-of-two range scale per token block.  W16 = fp16(s_w W) is an exact copy of the bf16 weight.
// The generated token's own logit, dz_y = g (1 - softmax_y), dominates each token's gradient and
// is kept out of the rounded operands altogether: its two rank-one terms, dz_y W_y into d_hidden
// and dz_y h_t into row y of d_w_lm, are added in fp32 by two small kernels (exact bf16 products,
// fixed summation order, no atomics).
//
// The first operand ("A role") indexes accumulator rows: a lane of the 32x32 MFMA result holds one
// column j and rows 8b + 4(lane/32) + c, so the reduction over the vocabulary in the forward pass
// is almost entirely inside a lane, and the gradient tiles store four consecutive k per lane.
//
// Workgroup: 256 threads = 4 waves as 2x2, each wave a 128x128 sub-tile (4x4 MFMA blocks, 256
// accumulator registers).  K is walked in tiles of 32 through a ring of four LDS stages of
// 2 x 16 KiB, filled by direct-to-LDS global loads three tiles ahead (see k_loop).
// Workgroup ids are mapped to tiles so that the 32 workgroups resident on one XCD (one L2) form a
// 4 x 8 block of tiles and share operand rows.
#include "loss.h"
#include "tile_map.h"

namespace pods {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;                            // k per LDS stage
constexpr int kOperandBytes = kTile * kBK * 2;     // 16 KiB: 256 rows x 64 B
constexpr int kStageBytes = 2 * kOperandBytes;     // A then B
constexpr int kStages = 4;                         // ring of LDS stages
constexpr int kDist = kStages - 1;                 // k-tiles in flight ahead of the one being multiplied
constexpr int kLdsBytes = kStages * kStageBytes;   // 128 KiB
constexpr int kQPitch = 2 * kTile + 8;             // bytes per token row of the q tile staged in LDS
constexpr int kStatsOffset = kTile * kQPitch > kLdsBytes ? kTile * kQPitch : kLdsBytes;   // past the staged q tile
constexpr int kFwdLdsBytes = kStatsOffset + 2 * 2 * kTile * 4;   // + [2][256] maxima and [2][256] sums: 134 KiB
constexpr int kHPitch = 4 * kTile + 16;            // bytes per token row of the d_hidden half-tile staged in LDS
constexpr int kDhLdsBytes = 128 * kHPitch > kLdsBytes ? 128 * kHPitch : kLdsBytes;   // 130 KiB
constexpr float kLog2e = 1.4426950408889634f;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// global_load_lds_dwordx4: each lane fetches 16 B from its own global address; the wave's 64 x 16 B
// land at consecutive LDS addresses starting at `lds_dst` (wave-uniform, carried in M0).  Issued as
// inline assembly so that the compiler does not pair it with the LDS reads it schedules (it would
// drain the whole vector-memory queue before each of them); completion is tracked by hand with
// s_waitcnt vmcnt.
// The global address is a wave-uniform base (a scalar register pair, advanced once per k-tile by two scalar
// additions) plus the lane's fixed 32-bit offset: no vector arithmetic per load.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds_16(uint64_t base, unsigned offset, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(offset), "s"(base)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt vmcnt(N), leaving expcnt and lgkmcnt alone (gfx9 encoding).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// Global -> LDS without passing through registers (global_load_lds_dwordx4): one wave instruction
// deposits 64 lanes x 16 B at consecutive LDS addresses, i.e. 16 rows of a 64-byte-row tile.  Lane l
// of wave w, instruction i fills row 64 i + 16 w + l/4, slot l%4, and therefore fetches the granule
// (l%4) ^ ((row >> 2) & 3) of that row: the XOR swizzle that makes the later ds_read_b128 fragment
// loads (16 consecutive rows, one granule column per pass) hit 16 distinct bank groups.
struct Operand {  // one operand's k-tiles: wave-uniform base of the current k-tile, this thread's 4 byte offsets
    uint64_t base;
    unsigned off[4];
    int64_t step;   // bytes from one k-tile to the next
};

__device__ __forceinline__ uint64_t uniform_address(const void* p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// Operand stored with the contraction index contiguous ("row-major rows x k"): tile = 256 rows x
// 64 B.  Rows at or beyond `rows` are clamped to the last row (their products are masked or
// multiplied by zeros by the caller).  Offsets are relative to row `row0`: at most 256 rows of ld elements
// (below 2^32 bytes for every supported shape).
__device__ __forceinline__ void operand_rows(Operand& op, const uint16_t* base, int64_t ld,
                                             int64_t row0, int64_t rows, int64_t col0) {
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int gc = (l & 3) ^ ((l >> 4) & 3);
    op.base = uniform_address(base + row0 * ld + col0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t row = row0 + 64 * i + 16 * w + (l >> 2);
        if (row >= rows) row = rows - 1;
        op.off[i] = (unsigned)(((row - row0) * ld + gc * 8) * 2);
    }
    op.step = 64;
}

// Operand stored with the contraction index as the ROW index ("k x columns", columns contiguous):
// tile = 32 k-rows x 256 columns (512 B per row); it is read back through the transposing LDS load
// (ds_read_b64_tr_b16), so no transposed copy of the matrix is ever made.  One wave instruction
// deposits two rows; lane l of wave w, instruction i fills row 8i + 2w + l/32, slot l%32, and
// fetches the granule (l%32) ^ ((row & 3) << 2): four consecutive k-rows then sit in four different
// 64-byte bank quarters, which is what the transposing read touches at once.
// Columns at or beyond `cols` (a multiple of 8) are clamped to the last granule (masked by the caller).
__device__ __forceinline__ void operand_kmajor(Operand& op, const uint16_t* base, int64_t ld,
                                               int64_t k0, int64_t col0, int64_t cols) {
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    op.base = uniform_address(base + k0 * ld + col0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 8 * i + 2 * w + (l >> 5);
        const int gc = (l & 31) ^ ((row & 3) << 2);
        int64_t col = col0 + gc * 8;
        if (col > cols - 8) col = cols - 8;
        op.off[i] = (unsigned)((row * ld + (col - col0)) * 2);
    }
    op.step = 32 * ld * 2;
}

struct LaneGeom {
    int a_rd, b_rd;   // row-major operands: LDS byte offset of this lane's fragment row (first block)
    int cx16;         // ... and the swizzle term of its fragment granule
    int a_km, b_km;   // k-major operands: LDS byte offset of this lane's transposing-read source
    int e6;           // ... and its swizzle term ((k row & 3) << 6)
    int wm, wn;       // wave position in the 2x2 wave grid
    int lane, wave;
};

__device__ __forceinline__ LaneGeom lane_geom() {
    LaneGeom g;
    const int tid = threadIdx.x;
    g.lane = tid & 63;
    g.wave = tid >> 6;
    g.wm = g.wave >> 1;
    g.wn = g.wave & 1;
    g.a_rd = (g.wm * 128 + (g.lane & 31)) * 64;
    g.b_rd = kOperandBytes + (g.wn * 128 + (g.lane & 31)) * 64;
    g.cx16 = ((g.lane >> 5) ^ ((g.lane >> 2) & 3)) << 4;
    // transposing read: within a block of 16 lanes, source lane j = 4e + q supplies 4 consecutive
    // columns of k-row e; result lane i receives column i of rows e = 0..3
    const int blk = g.lane >> 4, kg = blk >> 1, e = (g.lane >> 2) & 3, q = g.lane & 3;
    const int km = (kg * 8 + e) * 512 + (q & 1) * 8 + ((blk & 1) * 2 + (q >> 1)) * 16;
    g.a_km = km + g.wm * 256;
    g.b_km = kOperandBytes + km + g.wn * 256;
    g.e6 = e << 6;
    return g;
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma(f16x8 a, f16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;

// Fragment (32 rows x 16 k, 8 elements per lane) of MFMA block `blk`, k-step `ks`, from a stage.
template <typename E, bool KM>
__device__ __forceinline__ E read_frag(const unsigned char* stage, int rd, int km, int e6, int cx16,
                                       int blk, int ks) {
    if constexpr (!KM) {
        return *reinterpret_cast<const E*>(stage + rd + blk * 2048 + ((ks * 32) ^ cx16));
    } else {
        const unsigned char* p = stage + km + (e6 ^ (blk << 6)) + ks * 8192;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p + 2048));
        const i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(E, both);
    }
}

// acc += A . B^T over KT k-tiles of 32.  E is the operand element vector (bf16x8 or f16x8); AKM / BKM say
// which operands are k-major (see Operand).
//
// Each k-tile (two MFMA k-steps) lives in one stage of a ring of kStages LDS stages; kDist tiles
// are always in flight.  One iteration multiplies tile kt in two phases of 16 MFMAs:
//   phase 0: MFMAs on fragment set F0 (k-step 0, read during the previous iteration), interleaved
//            with the 8 direct-to-LDS loads of tile kt+kDist (into the stage consumed in the
//            previous iteration) and the fragment reads of F1 (k-step 1);
//   then     wait until this wave's share of tile kt+1 has landed, workgroup barrier;
//   phase 1: MFMAs on F1, interleaved with the fragment reads of tile kt+1's F0.
// The interleaving is pinned with scheduling barriers: left alone, the compiler issues the loads
// back to back, and the matrix pipe idles while the vector-memory queue drains.
// Every load that is issued is of a tile that will be multiplied: the last kDist tiles run in a tail
// loop that loads nothing.  (One branch-free body that kept loading past the end, into stages nobody
// reads, fetched 3 tiles too many per output tile: 5 % of the traffic and of the time when K is only
// 64 tiles, as in the logits.)
// On return nothing is in flight and the LDS ring may be reused after a barrier.
template <typename E, bool AKM, bool BKM, bool LOAD>
__device__ __forceinline__ void k_step(Operand& A, Operand& B, const unsigned char* cur, const unsigned char* nxt,
                                       unsigned dsta, const LaneGeom& g, E (&fa)[2][4],
                                       E (&fb)[2][4], f32x16 (&acc)[4][4]) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        { const int mi = (2 * i) >> 2, ni = (2 * i) & 3; acc[mi][ni] = mfma(fa[0][mi], fb[0][ni], acc[mi][ni]); }
        if constexpr (LOAD) {
            if (i < 4) load_to_lds_16(A.base, A.off[i], dsta + i * 4096);
            else load_to_lds_16(B.base, B.off[i - 4], dsta + kOperandBytes + (i - 4) * 4096);
            if (i == 3) A.base += A.step;
            if (i == 7) B.base += B.step;
        }
        __builtin_amdgcn_sched_barrier(0);
        { const int mi = (2 * i + 1) >> 2, ni = (2 * i + 1) & 3; acc[mi][ni] = mfma(fa[0][mi], fb[0][ni], acc[mi][ni]); }
        // all of F1 is requested in the first four slots (in the order phase 1 consumes it), so that
        // the wait before the barrier finds it long since delivered
        if (i == 0) { fa[1][0] = read_frag<E, AKM>(cur, g.a_rd, g.a_km, g.e6, g.cx16, 0, 1);
                      fb[1][0] = read_frag<E, BKM>(cur, g.b_rd, g.b_km, g.e6, g.cx16, 0, 1); }
        if (i == 1) { fb[1][1] = read_frag<E, BKM>(cur, g.b_rd, g.b_km, g.e6, g.cx16, 1, 1);
                      fb[1][2] = read_frag<E, BKM>(cur, g.b_rd, g.b_km, g.e6, g.cx16, 2, 1); }
        if (i == 2) { fb[1][3] = read_frag<E, BKM>(cur, g.b_rd, g.b_km, g.e6, g.cx16, 3, 1);
                      fa[1][1] = read_frag<E, AKM>(cur, g.a_rd, g.a_km, g.e6, g.cx16, 1, 1); }
        if (i == 3) { fa[1][2] = read_frag<E, AKM>(cur, g.a_rd, g.a_km, g.e6, g.cx16, 2, 1);
                      fa[1][3] = read_frag<E, AKM>(cur, g.a_rd, g.a_km, g.e6, g.cx16, 3, 1); }
        __builtin_amdgcn_sched_barrier(0);
    }
    // loads return in order: with loads still being issued, everything but the newest kDist-1 tiles is
    // in LDS; in the tail everything is waited for
    if constexpr (LOAD) wait_vmcnt<8 * (kDist - 1)>();
    else wait_vmcnt<0>();
    wait_lgkmcnt0();                 // this wave's reads of `cur` are done before others may refill it
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        { const int mi = (2 * i) >> 2, ni = (2 * i) & 3; acc[mi][ni] = mfma(fa[1][mi], fb[1][ni], acc[mi][ni]); }
        { const int mi = (2 * i + 1) >> 2, ni = (2 * i + 1) & 3; acc[mi][ni] = mfma(fa[1][mi], fb[1][ni], acc[mi][ni]); }
        if (i == 0) { fa[0][0] = read_frag<E, AKM>(nxt, g.a_rd, g.a_km, g.e6, g.cx16, 0, 0);
                      fb[0][0] = read_frag<E, BKM>(nxt, g.b_rd, g.b_km, g.e6, g.cx16, 0, 0); }
        if (i == 1) { fb[0][1] = read_frag<E, BKM>(nxt, g.b_rd, g.b_km, g.e6, g.cx16, 1, 0);
                      fb[0][2] = read_frag<E, BKM>(nxt, g.b_rd, g.b_km, g.e6, g.cx16, 2, 0); }
        if (i == 2) { fb[0][3] = read_frag<E, BKM>(nxt, g.b_rd, g.b_km, g.e6, g.cx16, 3, 0);
                      fa[0][1] = read_frag<E, AKM>(nxt, g.a_rd, g.a_km, g.e6, g.cx16, 1, 0); }
        if (i == 3) { fa[0][2] = read_frag<E, AKM>(nxt, g.a_rd, g.a_km, g.e6, g.cx16, 2, 0);
                      fa[0][3] = read_frag<E, AKM>(nxt, g.a_rd, g.a_km, g.e6, g.cx16, 3, 0); }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <typename E, bool AKM = false, bool BKM = false>
__device__ __forceinline__ void k_loop(Operand& A, Operand& B, int KT, unsigned char* lds,
                                       const LaneGeom& g, f32x16 (&acc)[4][4]) {
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)(lds + g.wave * 1024));
    E fa[2][4], fb[2][4];
    __builtin_amdgcn_s_barrier();   // every wave has left the ring (previous use)
    const int ahead = KT < kDist ? KT : kDist;   // tiles requested before the first one is multiplied
#pragma unroll
    for (int t = 0; t < kDist; ++t) {
        if (t < ahead) {
            const unsigned dsta = wave_lds + t * kStageBytes;
#pragma unroll
            for (int i = 0; i < 4; ++i) load_to_lds_16(A.base, A.off[i], dsta + i * 4096);
            A.base += A.step;
#pragma unroll
            for (int i = 0; i < 4; ++i) load_to_lds_16(B.base, B.off[i], dsta + kOperandBytes + i * 4096);
            B.base += B.step;
        }
    }
    if (KT >= kDist) wait_vmcnt<8 * (kDist - 1)>();   // the first tile is in
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[0][i] = read_frag<E, AKM>(lds, g.a_rd, g.a_km, g.e6, g.cx16, i, 0);
        fb[0][i] = read_frag<E, BKM>(lds, g.b_rd, g.b_km, g.e6, g.cx16, i, 0);
    }
    int kt = 0;
    // Four k-tiles per trip, one per stage of the ring, so that every stage address in the body is a constant
    // (the tile multiplied sits in stage s, the one requested goes into stage s - 1, consumed in the previous
    // step): LDS read addresses then need no arithmetic in the loop.
    for (; kt + kDist + kStages <= KT; kt += kStages) {
#pragma unroll
        for (int st = 0; st < kStages; ++st) {
            const int stn = (st + 1) % kStages, fill = (st + kDist) % kStages;
            k_step<E, AKM, BKM, true>(A, B, lds + st * kStageBytes, lds + stn * kStageBytes, wave_lds + fill * kStageBytes,
                                      g, fa, fb, acc);
        }
    }
    int st = 0;
    for (; kt + kDist < KT; ++kt) {   // what is left of the tiles that still request one
        const int stn = (st + 1 == kStages) ? 0 : st + 1;
        const int fill = (st + kDist) % kStages;
        k_step<E, AKM, BKM, true>(A, B, lds + st * kStageBytes, lds + stn * kStageBytes, wave_lds + fill * kStageBytes, g,
                                  fa, fb, acc);
        st = stn;
    }
    for (; kt < KT; ++kt) {           // the last tiles: nothing left to request
        const int stn = (st + 1 == kStages) ? 0 : st + 1;
        k_step<E, AKM, BKM, false>(A, B, lds + st * kStageBytes, lds + stn * kStageBytes, 0u, g, fa, fb, acc);
        st = stn;
    }
    wait_lgkmcnt0();
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[4][4]) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.0f;
}

// Accumulator element (mi, r) of a lane sits at row mi*32 + 8*(r/4) + 4*(lane/32) + r%4 of the
// wave's 128-row sub-tile.  Inverse for one row offset `rel` (relative to the sub-tile, already
// reduced by 4*(lane/32)): register index mi*16 + r, or -1 if this lane does not hold it.
__device__ __forceinline__ int acc_slot_of(int rel) {
    if (rel < 0 || rel >= 128 || (rel & 4) != 0) return -1;
    return ((rel >> 5) << 4) | (((rel >> 3) & 3) << 2) | (rel & 3);
}

// ------------------------------------------------------------------------------------------
// Forward: one workgroup per (token tile, vocabulary tile).  Per token: an integer exponent E (without
// `efix`, the smallest with 2^E >= exp(largest logit of the tile); with it, the token's agreed exponent
// efix[p] unless the tile's own lies two or more above), the sum of exp(z) 2^-E over the tile (one partial per
// vocabulary tile, merged later by the log-sum-exp kernel), z_y, and the tile's softmax numerators
// 2^14 exp(z) 2^-E <= 2^15 rounded to fp16 (0 at v = y and past V), token-major, into the block's q array.
// E is common to the tile's two vocabulary waves (exchanged through LDS).  Once the token's log-sum-exp is
// known, the numerators are 2^14 softmax up to one power of two per (token, vocabulary tile), which the
// normalising pass applies where it is not 1 (exact in fp16), and one factor per token, which the gradient
// kernels get with the token's weight.
// One tile per workgroup (rather than a workgroup walking many vocabulary tiles) keeps the 32
// workgroups of an XCD in step, which is what lets them share operand tiles in the 4 MiB L2.
// A launch covers the token tiles of one token block (first row row0) and vocabulary tiles
// vt0 .. vt0 + nvt_launch - 1.
// ------------------------------------------------------------------------------------------
template <bool PARTIAL>
__device__ __forceinline__ void fwd_epilogue(const f32x16 (&acc)[4][4], const LaneGeom& g, unsigned char* lds,
                                             const int32_t* __restrict__ tok, int64_t n_valid, int64_t gt,
                                             int64_t vt, int V, int64_t slot_stride,
                                             const float* __restrict__ efix, float* __restrict__ pmax,
                                             float* __restrict__ psum, float* __restrict__ zy,
                                             _Float16* __restrict__ qtile, int64_t ldq) {
    const int vtile = g.wm * 128 + 4 * (g.lane >> 5);        // tile-local vocabulary row of (mi=0, r=0)
    const int vbase = (int)vt * kTile + vtile;
    const int vlimit = V - vbase;                            // rows at or past this offset do not exist
    float* red_max = reinterpret_cast<float*>(lds + kStatsOffset);   // [2 vocabulary waves][256 tokens]
    float* red_sum = red_max + 2 * kTile;
    constexpr float kLog2Q = 14.0f;
    static_assert(kQScale == 16384.0f, "kLog2Q must be log2(kQScale)");
    float Mt[4], S[4];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        float m = -__builtin_huge_valf();
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (PARTIAL && mi * 32 + 8 * (r >> 2) + (r & 3) >= vlimit) continue;
                m = fmaxf(m, acc[mi][ni][r]);
            }
        m = fmaxf(m, __shfl_xor(m, 32, 64));          // lanes l and l^32: same token, other rows
        Mt[ni] = m;
        if (g.lane < 32) red_max[g.wm * kTile + g.wn * 128 + ni * 32 + g.lane] = m;
    }
    __syncthreads();
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {   // the tile holds at least one vocabulary row, so this is finite
        const float m = fmaxf(Mt[ni], red_max[(g.wm ^ 1) * kTile + g.wn * 128 + ni * 32 + (g.lane & 31)]);
        float e = ceilf(m * kLog2e);   // the tile's own exponent: an integer, 2^e >= exp(m) > 2^(e-1)
        if (efix != nullptr) {         // the token's agreed exponent serves unless this tile lies too far above it
            const int64_t p = gt * kTile + g.wn * 128 + ni * 32 + (g.lane & 31);
            const float ef = p < n_valid ? efix[p] : e;
            if (e <= ef + 1.0f) e = ef;
        }
        Mt[ni] = e;                    // the tile's reference exponent E: exp(m) <= 2^(E+1)
    }

    // The q tile goes to memory through LDS: a lane holds 4 consecutive vocabulary entries of one token,
    // so storing from registers would scatter 8-byte pieces over 32 token rows per instruction; staged
    // as [token][vocabulary] rows (pitch 520 B: the 32 rows a half-wave writes fall into 32 different
    // bank pairs) every later store instruction covers two whole 512-byte rows.
    // Two passes over the tile's tokens (MFMA block columns 0-1, then 2-3 of each wave): the stores of the
    // first pass drain while the second pass computes its exponentials.
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) {
            const int ni = 2 * pass + nj;
            const int tloc = g.wn * 128 + ni * 32 + (g.lane & 31);
            const int64_t p = gt * kTile + tloc;
            const bool valid = p < n_valid;
            // kQScale exp(z) 2^-E = 2^(z log2e - E + 14), at most 2^15; rows past N get 2^-inf = 0
            const float off = valid ? kLog2Q - Mt[ni] : -__builtin_huge_valf();
            unsigned char* row = lds + tloc * kQPitch + vtile * 2;
            float sum = 0.0f;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    f16x4 pk;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float e = __builtin_amdgcn_exp2f(fmaf(acc[mi][ni][b * 4 + c], kLog2e, off));
                        if (PARTIAL && mi * 32 + 8 * b + c >= vlimit) e = 0.0f;
                        sum += e;
                        pk[c] = (_Float16)e;
                    }
                    *reinterpret_cast<f16x4*>(row + (mi * 32 + 8 * b) * 2) = pk;
                }
            sum += __shfl_xor(sum, 32, 64);
            S[ni] = sum;
            // z_y lives in exactly one lane of one wave of one vocabulary tile; its numerator stays in the
            // sum and leaves q (the y logit's gradient is applied in fp32)
            const int y = valid ? tok[p] : -1;
            const int slot = acc_slot_of(y - vbase);
            if (__any(slot >= 0)) {
                float zv = 0.0f;
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (slot == mi * 16 + r) zv = acc[mi][ni][r];
                if (slot >= 0) {
                    zy[p] = zv;
                    *reinterpret_cast<_Float16*>(row + (y - vbase) * 2) = (_Float16)0.0f;
                }
            }
        }
        __syncthreads();
        // this pass filled token rows 128 h + 64 pass .. + 63 (h = 0, 1); wave w stores 32 of them, two rows
        // (2 x 512 B) per instruction
#pragma unroll 4
        for (int i = 0; i < 16; ++i) {
            const int r = (g.wave >> 1) * 128 + pass * 64 + (g.wave & 1) * 32 + 2 * i + (g.lane >> 5);
            const unsigned char* src = lds + r * kQPitch + (g.lane & 31) * 16;
            const f16x4 lo = *reinterpret_cast<const f16x4*>(src);
            const f16x4 hi = *reinterpret_cast<const f16x4*>(src + 8);
            const f16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            // streamed past the L2, whose lines are better spent on the operand tiles the XCD's workgroups share
            __builtin_nontemporal_store(both, reinterpret_cast<f16x8*>(qtile + (int64_t)r * ldq + (g.lane & 31) * 8));
        }
    }
    if (g.wm == 1 && g.lane < 32) {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) red_sum[g.wn * 128 + ni * 32 + g.lane] = S[ni];
    }
    __syncthreads();
    if (g.wm == 0 && g.lane < 32) {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const int tloc = g.wn * 128 + ni * 32 + g.lane;
            const int64_t p = gt * kTile + tloc;
            if (p < n_valid) {
                pmax[vt * slot_stride + p] = Mt[ni];
                psum[vt * slot_stride + p] = (S[ni] + red_sum[tloc]) * (1.0f / kQScale);
            }
        }
    }
}

__global__ __launch_bounds__(256, 1) void fwd_kernel(const LossHeader* __restrict__ hdr,
                                                     const int32_t* __restrict__ tok,
                                                     const uint16_t* __restrict__ ht,
                                                     const uint16_t* __restrict__ wt,
                                                     int d, int V, int vt0, int nvt_launch, int64_t row0,
                                                     int ntt_grid, int64_t slot_stride,
                                                     const float* __restrict__ efix,
                                                     float* __restrict__ pmax, float* __restrict__ psum,
                                                     float* __restrict__ zy, int64_t ldq,
                                                     _Float16* __restrict__ q) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int64_t n_valid = hdr->n_valid;
    int64_t tt, vt;
    if (!decode_tile(blockIdx.x, ntt_grid, nvt_launch, tt, vt)) return;
    const int64_t gt = row0 / kTile + tt;         // token tile among all packed rows
    if (gt * kTile >= n_valid) return;
    vt += vt0;
    const LaneGeom g = lane_geom();
    const int KT = d / kBK;

    Operand A, B;
    operand_kmajor(A, wt + vt * d * kTile, kTile, 0, 0, kTile);
    operand_kmajor(B, ht + gt * d * kTile, kTile, 0, 0, kTile);
    f32x16 acc[4][4];
    zero_acc(acc);
    k_loop<bf16x8, true, true>(A, B, KT, lds, g, acc);

    __builtin_amdgcn_s_barrier();                 // every wave has left the operand ring
    _Float16* qtile = q + (tt * kTile) * ldq + vt * kTile;
    if ((int)vt * kTile + kTile > V)              // last vocabulary tile: rows >= V do not exist
        fwd_epilogue<true>(acc, g, lds, tok, n_valid, gt, vt, V, slot_stride, efix, pmax, psum, zy, qtile, ldq);
    else
        fwd_epilogue<false>(acc, g, lds, tok, n_valid, gt, vt, V, slot_stride, efix, pmax, psum, zy, qtile, ldq);
}

// ------------------------------------------------------------------------------------------
// The exponent a token's vocabulary tiles agree on, fixed after the block's first forward launch: four above the
// larger of (a) the exponents of that launch's `slots0` tiles and (b) that of the generated token's own logit
// z_y = h_t . W_y (fp32 dot product of the bf16 rows; only its binade matters here).  One wave per token.
// ------------------------------------------------------------------------------------------
// (The margin costs nothing in precision: the largest numerator of a token keeps all its bits, and fp16 still holds
// full precision 24 binades below 2^14 2^-margin, i.e. down to softmax terms e^-16 of the largest.)
constexpr float kExponentMargin = 4.0f;
__global__ __launch_bounds__(256) void exponent_kernel(const LossHeader* __restrict__ hdr,
                                                       const int32_t* __restrict__ row_map,
                                                       const int32_t* __restrict__ tok,
                                                       const uint16_t* __restrict__ hidden,
                                                       const uint16_t* __restrict__ w, int d,
                                                       const float* __restrict__ pmax, int slots0,
                                                       int64_t slot_stride, int64_t row0, int64_t row_end,
                                                       float* __restrict__ efix) {
    const int lane = threadIdx.x & 63;
    const int64_t p = row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= hdr->n_valid || p >= row_end) return;
    const uint16_t* h = hidden + (int64_t)row_map[p] * d;
    const uint16_t* wy = w + (int64_t)tok[p] * d;
    float dot = 0.0f;
    for (int k = lane * 8; k < d; k += 512) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(h + k);
        const u32x4 y = *reinterpret_cast<const u32x4*>(wy + k);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dot = fmaf(__uint_as_float(x[j] << 16), __uint_as_float(y[j] << 16), dot);
            dot = fmaf(__uint_as_float(x[j] & 0xFFFF0000u), __uint_as_float(y[j] & 0xFFFF0000u), dot);
        }
    }
    float m = -__builtin_huge_valf();
    for (int s = lane; s < slots0; s += 64) m = fmaxf(m, pmax[s * slot_stride + p]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        dot += __shfl_xor(dot, o, 64);
        m = fmaxf(m, __shfl_xor(m, o, 64));
    }
    if (lane == 0) efix[p] = fmaxf(m, ceilf(dot * kLog2e)) + kExponentMargin;
}

// ------------------------------------------------------------------------------------------
// Normalise (per token block, once its log-sum-exp is known): the forward pass's numerators times the power
// of two of their (token, vocabulary tile), in place: exact in fp16 (results below 2^-24 vanish).  Afterwards
// q = 2^14 softmax / c_t with the per-token factor c_t that rides on the token's weight.  A factor of 1
// (the tile was written under the token's final exponent) leaves the tile untouched.  One workgroup per
// (8 vocabulary tiles, 32 token rows): it leaves at once when all its 256 factors are 1; otherwise it walks its
// rows, 16 bytes per lane and 4 KiB contiguous per row.  Bound by HBM (2 x 2 bytes per logit it touches).
// ------------------------------------------------------------------------------------------
constexpr int kRescaleRows = 32;
__global__ __launch_bounds__(256) void rescale_kernel(const LossHeader* __restrict__ hdr,
                                                      const _Float16* __restrict__ qscale, int64_t slot_stride,
                                                      int64_t row0, int ntiles, int64_t ldq,
                                                      _Float16* __restrict__ q) {
    __shared__ _Float16 sc[8][kRescaleRows];
    const int64_t r0 = (int64_t)blockIdx.y * kRescaleRows;
    const int64_t n_bwd = hdr->n_bwd;
    if (row0 + r0 >= n_bwd) return;
    const int tile0 = blockIdx.x * 8;
    {
        const int tl = threadIdx.x >> 5, rl = threadIdx.x & 31;      // 8 tiles x 32 rows
        _Float16 s = (_Float16)1.0f;
        if (tile0 + tl < ntiles && row0 + r0 + rl < n_bwd) s = qscale[(int64_t)(tile0 + tl) * slot_stride + row0 + r0 + rl];
        sc[tl][rl] = s;
        if (__syncthreads_or(s != (_Float16)1.0f) == 0) return;
    }
    const int tl = threadIdx.x >> 5;                                 // 32 granules of 8 per vocabulary tile
    if (tile0 + tl >= ntiles) return;
    _Float16* at = q + r0 * ldq + (int64_t)tile0 * kTile + (int64_t)threadIdx.x * 8;
#pragma unroll 4
    for (int r = 0; r < kRescaleRows; ++r) {
        const _Float16 s = sc[tl][r];
        if (s != (_Float16)1.0f) {
            f16x8 x = *reinterpret_cast<const f16x8*>(at + r * ldq);
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = x[j] * s;
            *reinterpret_cast<f16x8*>(at + r * ldq) = x;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Backward: d_hidden[t][k] -= (g_t / (kQScale s_w)) sum_v q[t][v] W16[v][k], W16 = s_w W, over the whole
// vocabulary, for the token tiles of one token block (the rows were initialised with the y-logit term)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void dh_kernel(const LossHeader* __restrict__ hdr,
                                                    const int32_t* __restrict__ row_map,
                                                    const float* __restrict__ gvec,
                                                    const uint16_t* __restrict__ w16,
                                                    const uint16_t* __restrict__ q, int64_t ldq, int d,
                                                    int dk, int V, int64_t row0, int ntt_grid,
                                                    float* __restrict__ d_hidden) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int64_t n_valid = hdr->n_bwd;
    int64_t tb, kt0;      // token tile within the block, d-tile
    if (!decode_tile(blockIdx.x, ntt_grid, (d + kTile - 1) / kTile, tb, kt0)) return;
    const int64_t tt = row0 / kTile + tb;             // token tile among all packed rows
    if (tt * kTile >= n_valid) return;
    const LaneGeom g = lane_geom();

    Operand A, B;
    operand_kmajor(A, w16, dk, 0, kt0 * kTile, dk);  // rows v >= V and columns k >= d of W16 are zero
    // every row of a token tile that holds a valid row was written by the forward step (zeros past N)
    operand_rows(B, q, ldq, tb * kTile, (tb + 1) * kTile, 0);
    f32x16 acc[4][4];
    zero_acc(acc);
    const int vwidth = (V + kTile - 1) / kTile * kTile;   // whole tiles that hold vocabulary
    k_loop<f16x8, true, false>(A, B, vwidth / kBK, lds, g, acc);

    // The tile is added to d_hidden through LDS, half of its tokens at a time: a lane holds 4 consecutive
    // k of one token, so updating from registers would touch 32-byte pieces of 32 different rows per
    // instruction; staged as [token][k] rows (pitch 1040 B: the 8 rows one LDS write cycle covers fall
    // into different banks), every global load and store covers one whole 1 KiB row segment.
    const float wscale_inv = -1.0f / (kQScale * w_range_scale(hdr));
    for (int half = 0; half < 2; ++half) {
        __syncthreads();   // the ring (first pass) or the previous half has been consumed
        // wave w updates rows 32 w .. 32 w + 31 of this half in four batches of eight rows; a batch's
        // d_hidden values are requested one batch ahead (the first before the staging below), so that
        // their latency is covered by the staging and by the previous batch's additions and stores
        const int64_t p0 = tt * kTile + half * 128 + g.wave * 32;
        const int live = (int)(n_valid - p0 < 32 ? (n_valid - p0 < 0 ? 0 : n_valid - p0) : 32);   // rows are in token order
        const int my_row = (g.lane < live) ? row_map[p0 + g.lane] : 0;
        const int k = (int)kt0 * kTile + g.lane * 4;
        const bool cols = k < d;
        f32x4 cur[2][8];
        auto row_ptr = [&](int i) {   // row i of this wave's 32; past the end: the batch's first row
            const int src_lane = i < live ? i : (i & ~7);
            const int64_t row = __builtin_amdgcn_readlane(my_row, src_lane);
            return reinterpret_cast<f32x4*>(d_hidden + row * d + k);
        };
        if (cols && live > 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) cur[0][j] = *row_ptr(j);
        }
        if (g.wn == half) {
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int tloc = ni * 32 + (g.lane & 31);
                const int64_t p = tt * kTile + half * 128 + tloc;
                const float scale = (p < n_valid) ? gvec[p] * wscale_inv : 0.0f;
                unsigned char* row = lds + tloc * kHPitch + (g.wm * 128 + 4 * (g.lane >> 5)) * 4;
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        f32x4 v;
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = acc[mi][ni][b * 4 + c] * scale;
                        *reinterpret_cast<f32x4*>(row + (mi * 32 + 8 * b) * 4) = v;
                    }
            }
        }
        __syncthreads();
        if (cols) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (8 * b < live) {
                    if (b + 1 < 4 && 8 * (b + 1) < live) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) cur[(b + 1) & 1][j] = *row_ptr(8 * (b + 1) + j);
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (8 * b + j < live) {
                            const int r = g.wave * 32 + 8 * b + j;
                            const f32x4 v = *reinterpret_cast<const f32x4*>(lds + r * kHPitch + g.lane * 16);
                            *row_ptr(8 * b + j) = v + cur[b & 1][j];
                        }
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Backward: d_w_lm[v][k] (+)= -(1 / (kQScale s)) sum_{t in block} q[t][v] H16[t][k], H16 = s g_t h_t with the
// block's range scale s.  The first token block stores (or adds to the caller's array, when accumulating),
// the later ones add: the blocks are summed in their fixed order.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void dw_kernel(const LossHeader* __restrict__ hdr,
                                                    const uint32_t* __restrict__ gmax_block,
                                                    const uint16_t* __restrict__ h16,
                                                    const uint16_t* __restrict__ q, int64_t ldq,
                                                    int d, int dk, int V, int64_t row0, int64_t nb,
                                                    int first_block, int accumulate, int64_t wg0,
                                                    float* __restrict__ d_w) {
    extern __shared__ __align__(16) unsigned char lds[];
    int64_t n_rows = hdr->n_bwd - row0;               // rows of this block that take part
    n_rows = n_rows < 0 ? 0 : (n_rows > nb ? nb : n_rows);
    if (n_rows == 0 && !first_block) return;          // nothing to add
    const int64_t vround = ((int64_t)V + kTile - 1) / kTile * kTile;
    int64_t vt, kt0;
    const int64_t nvt = vround / kTile, ndt = (d + kTile - 1) / kTile;
    if (use_strips(nvt) ? !decode_strip_tile(wg0 + blockIdx.x, nvt, ndt, vt, kt0)
                        : !decode_tile(wg0 + blockIdx.x, nvt, ndt, vt, kt0))
        return;
    const LaneGeom g = lane_geom();

    Operand A, B;
    // token rows past N (up to the end of the last token tile) are zero in H16 and finite in q
    operand_kmajor(A, h16, dk, row0, kt0 * kTile, dk);
    operand_kmajor(B, q, ldq, 0, vt * kTile, vround);
    f32x16 acc[4][4];
    zero_acc(acc);
    const int KT = (int)((n_rows + kBK - 1) / kBK);
    if (KT > 0) k_loop<f16x8, true, true>(A, B, KT, lds, g, acc);
    const float scale = -1.0f / (kQScale * g_range_scale(*gmax_block, hdr));

#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        const int64_t v = vt * kTile + g.wn * 128 + ni * 32 + (g.lane & 31);
        if (v >= V) continue;
        float* row = d_w + v * d;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int k = (int)kt0 * kTile + g.wm * 128 + mi * 32 + 8 * b + 4 * (g.lane >> 5);
                if (k >= d) continue;
                f32x4 vv;
#pragma unroll
                for (int c = 0; c < 4; ++c) vv[c] = acc[mi][ni][b * 4 + c] * scale;
                if (accumulate) vv += *reinterpret_cast<const f32x4*>(row + k);
                *reinterpret_cast<f32x4*>(row + k) = vv;
            }
    }
}

// ------------------------------------------------------------------------------------------
// The generated token's own logit, in fp32.  coef_t = g_t (1 - softmax_y) = d loss / d z_y.
//   d_hidden[t][:]  = coef_t W[y_t][:]            (initialises the row; the contraction accumulates on it)
//   d_w_lm[y_t][:] += coef_t h_t[:]               (after the token blocks have stored and added their parts)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dh_onehot_kernel(const LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ row_map,
                                                        const int32_t* __restrict__ tok,
                                                        const float* __restrict__ coef,
                                                        const uint16_t* __restrict__ w, int d,
                                                        int64_t row0, float* __restrict__ d_hidden) {
    const int64_t p = row0 + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // one wave per token
    if (p >= hdr->n_bwd) return;
    const int lane = threadIdx.x & 63;
    const float c = coef[p];
    const uint16_t* wrow = w + (int64_t)tok[p] * d;
    float* out = d_hidden + (int64_t)row_map[p] * d;
    for (int k = lane * 8; k < d; k += 512) {   // d % 8 == 0: whole groups of 8
        const u32x4 raw = *reinterpret_cast<const u32x4*>(wrow + k);
        f32x4 lo, hi;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float e0 = __uint_as_float(raw[j] << 16), e1 = __uint_as_float(raw[j] & 0xFFFF0000u);
            if (j < 2) { lo[2 * j] = c * e0; lo[2 * j + 1] = c * e1; }
            else { hi[2 * j - 4] = c * e0; hi[2 * j - 3] = c * e1; }
        }
        *reinterpret_cast<f32x4*>(out + k) = lo;
        *reinterpret_cast<f32x4*>(out + k + 4) = hi;
    }
}

// One wave owns 64 consecutive vocabulary rows and walks every token in order; a row's terms are
// therefore added by the same lanes in ascending token order, whatever the timing.
constexpr int kOnehotRows = 64;
__global__ __launch_bounds__(256) void dw_onehot_kernel(const LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ row_map,
                                                        const int32_t* __restrict__ tok,
                                                        const float* __restrict__ coef,
                                                        const uint16_t* __restrict__ hidden, int d,
                                                        int V, float* __restrict__ d_w) {
    const int n_valid = hdr->n_bwd;
    const int lane = threadIdx.x & 63;
    const int v_lo = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kOnehotRows;
    if (v_lo >= V) return;
    constexpr int kAhead = 8;     // token ids are fetched 8 x 64 at a time: the scan is bound by their latency
    for (int q0 = 0; q0 < n_valid; q0 += 64 * kAhead) {
        int ys[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            const int p = q0 + i * 64 + lane;
            ys[i] = (p < n_valid) ? tok[p] : -1;
        }
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            const int p0 = q0 + i * 64;
            const int y = ys[i];
            unsigned long long hits = __ballot((unsigned)(y - v_lo) < (unsigned)kOnehotRows);
            while (hits != 0ull) {
                const int src = __ffsll((long long)hits) - 1;
                hits &= hits - 1ull;
                const int pp = p0 + src;
                const int yy = __shfl(y, src, 64);
                const float c = coef[pp];
                if (c == 0.0f) continue;
                const uint16_t* hrow = hidden + (int64_t)row_map[pp] * d;
                float* out = d_w + (int64_t)yy * d;
                for (int k = lane * 8; k < d; k += 512) {
                    const u32x4 raw = *reinterpret_cast<const u32x4*>(hrow + k);
                    f32x4 lo = *reinterpret_cast<f32x4*>(out + k);
                    f32x4 hi = *reinterpret_cast<f32x4*>(out + k + 4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float e0 = __uint_as_float(raw[j] << 16), e1 = __uint_as_float(raw[j] & 0xFFFF0000u);
                        if (j < 2) { lo[2 * j] += c * e0; lo[2 * j + 1] += c * e1; }
                        else { hi[2 * j - 4] += c * e0; hi[2 * j - 3] += c * e1; }
                    }
                    *reinterpret_cast<f32x4*>(out + k) = lo;
                    *reinterpret_cast<f32x4*>(out + k + 4) = hi;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Transposed bf16 operand copies for the logits contraction (once per call), so that it too reads
// k-major tiles (512 contiguous bytes per k-row instead of 64):
//   Wt[v/256][k][v%256] = W[v][k]            (zero for v >= V up to the end of the last tile)
//   Ht[p/256][k][p%256] = H[row_map[p]][k]   (zero for p >= N up to the end of the last tile)
// Blocked by 256-column tile, so that the k-tile a workgroup streams (32 k-rows x 512 B) is one
// contiguous 16 KiB run and a whole tile column is one contiguous d x 512 B region.
// The logits are multiplied in bf16, the inputs' own type: exact products either way, and under the
// chip's power limit the bf16 matrix instruction sustains 9 % more than the fp16 one (measured on an
// MFMA-only loop: 1.74 against 1.59 PFLOP/s).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void transpose_kernel(LossHeader* __restrict__ hdr,
                                                        const int32_t* __restrict__ gather,
                                                        const uint16_t* __restrict__ src, int64_t rows,
                                                        int d, int dk, int64_t rows_out, int token_rows,
                                                        uint16_t* __restrict__ dst) {
    // 64 rows x 64 k per workgroup, 16 bytes per lane both ways: a lane reads 8 consecutive k of one row,
    // scatters them into the transposed LDS tile, and later writes 8 consecutive rows of one k.
    constexpr int kPitch = 72;                         // halfwords per k-row of the tile: 16-byte aligned rows
    __shared__ __align__(16) uint16_t tile[64 * kPitch];
    int64_t nrows = rows, fill_to = rows_out;
    if (token_rows) {
        nrows = hdr->n_valid;
        fill_to = (nrows + kTile - 1) / kTile * kTile;
    }
    const int64_t r0 = (int64_t)blockIdx.x * 64;
    const int k0 = blockIdx.y * 64;
    if (r0 >= fill_to) return;
    const int sub = threadIdx.x & 7, line = threadIdx.x >> 3;   // 8 granules of 8 x 32 lines per pass
    uint32_t amax = 0u;   // largest |x| seen, as bf16 bits (non-negative floats order as integers)
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int rr = pass * 32 + line;
        const int64_t r = r0 + rr;
        const int k = k0 + sub * 8;                    // d is a multiple of 8: a granule lies inside the row or outside
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (r < nrows && k < d) {
            const int64_t srow = gather ? (int64_t)gather[r] : r;
            raw = *reinterpret_cast<const u32x4*>(src + srow * d + k);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = raw[j] & 0xFFFFu, hi = raw[j] >> 16;
            tile[(sub * 8 + 2 * j) * kPitch + rr] = (uint16_t)lo;
            tile[(sub * 8 + 2 * j + 1) * kPitch + rr] = (uint16_t)hi;
            amax = max(amax, max(lo & 0x7FFFu, hi & 0x7FFFu));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off, 64));
    if ((threadIdx.x & 63) == 0 && amax != 0u) {
        // a plain look first: after the first few workgroups nearly none still raises the maximum, and
        // hundreds of thousands of atomics on one address would take longer than the copy itself
        uint32_t* slot = token_rows ? &hdr->hmax_bits : &hdr->wmax_bits;
        if ((amax << 16) > *reinterpret_cast<volatile uint32_t*>(slot)) atomicMax(slot, amax << 16);
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int kk = pass * 32 + line;
        const int64_t r = r0 + sub * 8;                // 8 consecutive rows: inside one 256-row block of dst
        if (k0 + kk < dk && r < rows_out)              // k in [d, dk): zeros
            *reinterpret_cast<u32x4*>(dst + ((r / kTile) * dk + (k0 + kk)) * kTile + r % kTile) =
                *reinterpret_cast<const u32x4*>(&tile[kk * kPitch + sub * 8]);
    }
}

// ------------------------------------------------------------------------------------------
// fp16 operand copies:
//   W16[v][k] = s_w W[v][k]               (once per call; zero rows for v >= V; exact in fp16's normal range:
//                                          bf16 has fewer significand bits; s_w = the range scale of W)
//   H16[p][k] = s g_p H[row_map[p]][k]    (per token block, rows row0 .. row0 + rows - 1; zero rows for
//                                          p >= N up to the end of the last token tile; s = the block's
//                                          range scale of g)
// One thread per 8 elements.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void convert_kernel(const LossHeader* __restrict__ hdr,
                                                      const uint32_t* __restrict__ gmax_block,
                                                      const int32_t* __restrict__ gather,
                                                      const float* __restrict__ gvec,
                                                      const uint16_t* __restrict__ src, int64_t row0,
                                                      int64_t rows, int64_t rows_valid, int d, int dk,
                                                      int token_rows, _Float16* __restrict__ dst) {
    int64_t nrows = rows_valid, fill_to = row0 + rows;
    float common;
    if (token_rows) {
        nrows = hdr->n_bwd;
        const int64_t tile_end = (nrows + kTile - 1) / kTile * kTile;
        fill_to = tile_end < fill_to ? tile_end : fill_to;
        common = g_range_scale(*gmax_block, hdr);
    } else {
        common = w_range_scale(hdr);
    }
    const int per_row = dk / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = row0 + idx / per_row;
    const int k = (int)(idx % per_row) * 8;
    if (r >= fill_to) return;
    f16x8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = (_Float16)0.0f;
    if (r < nrows && k < d) {   // d is a multiple of 8: a granule lies inside the row or in the zero padding
        const int64_t srow = gather ? (int64_t)gather[r] : r;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(src + srow * d + k);
        const float sc = token_rows ? common * gvec[r] : common;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            out[2 * j] = (_Float16)(__uint_as_float(raw[j] << 16) * sc);
            out[2 * j + 1] = (_Float16)(__uint_as_float(raw[j] & 0xFFFF0000u) * sc);
        }
    }
    *reinterpret_cast<f16x8*>(dst + r * dk + k) = out;
}

pods_status reserve(const void* kernel, const char* what, int bytes = kLdsBytes) {
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return fail(PODS_ERR_RUNTIME, "%s: cannot reserve LDS: %s", what, hipGetErrorString(e));
    return PODS_OK;
}

}  // namespace

pods_status mfma_forward_backward(const LossArgs& a, const LossPlan& p) {
    unsigned char* ws = a.workspace;
    auto* hdr = reinterpret_cast<LossHeader*>(ws + p.off_hdr);
    auto* gmax = reinterpret_cast<const uint32_t*>(ws + p.off_gmax);
    auto* row_map = reinterpret_cast<const int32_t*>(ws + p.off_rowmap);
    auto* tok = reinterpret_cast<const int32_t*>(ws + p.off_tok);
    auto* lse = reinterpret_cast<const float*>(ws + p.off_lse);
    auto* g = reinterpret_cast<const float*>(ws + p.off_g);
    auto* coef = reinterpret_cast<const float*>(ws + p.off_coef);
    auto* pmax = reinterpret_cast<float*>(ws + p.off_pmax);
    auto* psum = reinterpret_cast<float*>(ws + p.off_psum);
    auto* zy = reinterpret_cast<float*>(ws + p.off_zy);
    auto* wt = reinterpret_cast<uint16_t*>(ws + p.off_wtt);
    auto* ht = reinterpret_cast<uint16_t*>(ws + p.off_htt);
    auto* w16 = reinterpret_cast<_Float16*>(ws + p.off_wt);
    auto* h16 = reinterpret_cast<_Float16*>(ws + p.off_ht);
    auto* q = reinterpret_cast<_Float16*>(ws + p.off_dz);
    auto* qscale = reinterpret_cast<const _Float16*>(ws + p.off_qscale);
    auto* efix = reinterpret_cast<float*>(ws + p.off_efix);
    const auto* hidden = static_cast<const uint16_t*>(a.hidden);
    const auto* w = static_cast<const uint16_t*>(a.w_lm);
    pods_status st;
    if ((st = reserve(reinterpret_cast<const void*>(fwd_kernel), "token loss forward", kFwdLdsBytes)) != PODS_OK) return st;
    if ((st = reserve(reinterpret_cast<const void*>(dh_kernel), "token loss d_hidden", kDhLdsBytes)) != PODS_OK) return st;
    if ((st = reserve(reinterpret_cast<const void*>(dw_kernel), "token loss d_w_lm")) != PODS_OK) return st;

    // once per call: transposed bf16 copies for the logits (they also find max |W|, max |h|), fp16 copy of W
    const unsigned dtiles64 = (unsigned)(p.dk / 64);
    PODS_LAUNCH("transpose W", a.stream, transpose_kernel, dim3((unsigned)(p.vld / 64), dtiles64), dim3(256), 0,
                a.stream, hdr, nullptr, w, (int64_t)a.V, a.d, p.dk, p.vld, 0, wt);
    if ((st = check_launch("transpose W")) != PODS_OK) return st;
    PODS_LAUNCH("transpose H", a.stream, transpose_kernel, dim3((unsigned)(p.ncap_ld / 64), dtiles64), dim3(256), 0,
                a.stream, hdr, row_map, hidden, (int64_t)0, a.d, p.dk, p.ncap_ld, 1, ht);
    if ((st = check_launch("transpose H")) != PODS_OK) return st;
    const int64_t per_row = p.dk / 8;
    PODS_LAUNCH("convert W", a.stream, convert_kernel, dim3((unsigned)ceil_div(p.vld * per_row, 256)), dim3(256), 0,
                a.stream, hdr, nullptr, nullptr, nullptr, w, (int64_t)0, p.vld, (int64_t)a.V, a.d, p.dk, 0, w16);
    if ((st = check_launch("convert W")) != PODS_OK) return st;

    const int64_t nvt = p.vld / kTile;
    const int64_t dt256 = ceil_div(a.d, kTile);
    const int64_t step_vt = kDefaultVocabChunk / kTile;
    for (int b = 0; b < p.nblocks; ++b) {
        const int64_t row0 = (int64_t)b * p.nb;
        const int64_t rows = p.ncap_ld - row0 < p.nb ? p.ncap_ld - row0 : p.nb;   // capacity of this block
        const int64_t ntt = rows / kTile;
        // Forward, one launch per kDefaultVocabChunk columns: the chunk of W then stays in the Infinity Cache
        // while the block's token tiles stream past it.
        for (int64_t vt0 = 0; vt0 < nvt; vt0 += step_vt) {
            const int64_t nl = nvt - vt0 < step_vt ? nvt - vt0 : step_vt;
            PODS_LAUNCH("token loss forward", a.stream, fwd_kernel, dim3((unsigned)super_grid_blocks(ntt, nl)),
                        dim3(256), kFwdLdsBytes, a.stream, hdr, tok, reinterpret_cast<const uint16_t*>(ht),
                        reinterpret_cast<const uint16_t*>(wt), p.dk, a.V, (int)vt0, (int)nl, row0, (int)ntt,
                        p.ncap_ld, vt0 == 0 ? static_cast<const float*>(nullptr) : efix, pmax, psum, zy, p.ldq, q);
            if ((st = check_launch("token loss forward")) != PODS_OK) return st;
            if (vt0 == 0 && nl < nvt) {   // later launches write under the exponent each token fixes now
                PODS_LAUNCH("token loss exponent", a.stream, exponent_kernel, dim3((unsigned)ceil_div(rows, 4)), dim3(256),
                            0, a.stream, hdr, row_map, tok, hidden, w, a.d, pmax, (int)nl, p.ncap_ld, row0, row0 + rows,
                            efix);
                if ((st = check_launch("token loss exponent")) != PODS_OK) return st;
            }
        }
        if ((st = launch_surrogate(a, p, row0, rows, b)) != PODS_OK) return st;
        PODS_LAUNCH("token loss normalise", a.stream, rescale_kernel,
                    dim3((unsigned)ceil_div(nvt, 8), (unsigned)ceil_div(rows, kRescaleRows)), dim3(256), 0, a.stream, hdr,
                    qscale, p.ncap_ld, row0, (int)nvt, p.ldq, q);
        if ((st = check_launch("token loss normalise")) != PODS_OK) return st;
        PODS_LAUNCH("convert H", a.stream, convert_kernel, dim3((unsigned)ceil_div(rows * per_row, 256)), dim3(256), 0,
                    a.stream, hdr, gmax + b, row_map, g, hidden, row0, rows, (int64_t)0, a.d, p.dk, 1, h16);
        if ((st = check_launch("convert H")) != PODS_OK) return st;
        PODS_LAUNCH("token loss d_hidden (y logit)", a.stream, dh_onehot_kernel, dim3((unsigned)ceil_div(rows, 4)),
                    dim3(256), 0, a.stream, hdr, row_map, tok, coef, w, a.d, row0, a.d_hidden);
        if ((st = check_launch("token loss d_hidden (y logit)")) != PODS_OK) return st;
        PODS_LAUNCH("token loss d_hidden", a.stream, dh_kernel, dim3((unsigned)super_grid_blocks(ntt, dt256)), dim3(256),
                    kDhLdsBytes, a.stream, hdr, row_map, g, reinterpret_cast<const uint16_t*>(w16),
                    reinterpret_cast<const uint16_t*>(q), p.ldq, a.d, p.dk, a.V, row0, (int)ntt, a.d_hidden);
        if ((st = check_launch("token loss d_hidden")) != PODS_OK) return st;
        // With many vocabulary tiles: one launch per round of the chip (see decode_strip_tile).
        const bool strips = use_strips(nvt);
        const int64_t dw_total = strips ? strip_grid_blocks(nvt, dt256) : super_grid_blocks(nvt, dt256);
        const int64_t dw_round = strips ? kRoundWorkgroups : dw_total;
        for (int64_t wg0 = 0; wg0 < dw_total; wg0 += dw_round) {
            const int64_t nwg = dw_total - wg0 < dw_round ? dw_total - wg0 : dw_round;
            PODS_LAUNCH("token loss d_w_lm", a.stream, dw_kernel, dim3((unsigned)nwg), dim3(256),
                        kLdsBytes, a.stream, hdr, gmax + b, reinterpret_cast<const uint16_t*>(h16),
                        reinterpret_cast<const uint16_t*>(q), p.ldq, a.d, p.dk, a.V, row0, rows, b == 0 ? 1 : 0,
                        (a.accumulate_d_w || b > 0) ? 1 : 0, wg0, a.d_w_lm);
        }
        if ((st = check_launch("token loss d_w_lm")) != PODS_OK) return st;
    }
    PODS_LAUNCH("token loss d_w_lm (y logit)", a.stream, dw_onehot_kernel, dim3((unsigned)ceil_div(a.V, 4 * kOnehotRows)), dim3(256), 0,
                       a.stream, hdr, row_map, tok, coef, hidden, a.d, a.V, a.d_w_lm);
    return check_launch("token loss d_w_lm (y logit)");
}

}  // namespace pods
