// bf16 MFMA GEMM for gfx950, C[M,N] = A[M,K] * B[N,K]^T with both operands K-contiguous,
// and the epilogues of the LM-head path fused onto its accumulators:
//   * vocabulary GEMM (rows = vocabulary entries, columns = tokens): running max / sum-exp per
//     token over the tile's vocabulary rows, so full logits never reach HBM; optionally the
//     chunk's exponentials against a per-token reference, or directly the softmax-gradient
//     entries, in bf16;
//   * plain stores (fp32 / bf16, overwrite or accumulate, optional row scatter) for dH and dW.
//
// One workgroup owns a BM x BN output tile. K is streamed in slices of BK elements that go from
// global memory straight into LDS (global_load_lds_dwordx4: no register staging, no ds_write),
// into one ring of slices per operand (the A ring may be one slice deeper). Each wavefront
// owns a (BM/WGM) x (BN/WGN) sub-tile of 16x16x32 MFMA blocks
// (with random operands the chip is power-limited, and a register-only loop of 16x16x32
// instructions sustains 15 % more than one of 32x32x16: 2.02 against 1.76 PFLOP/s) and reads its
// operands one 32-wide k-step ahead. The single barrier per slice sits before the LAST k-step of
// the slice: the first operands of the next slice are fetched, and the freed buffers are refilled,
// while the current slice still computes.
//
// LDS layout: a tile row is BK*2 bytes; its 16-byte chunks are XOR-swizzled so that the lanes a
// ds_read_b128 serves in one cycle fall into 16 different 16-byte bank groups of the 64-bank LDS.
// Measured with the bank-conflict counter: a ds_read_b128 is served 16 lanes per cycle, and the
// lanes that go together are {0-7, 24-31}, {8-15, 16-23}, {32-39, 56-63}, {40-47, 48-55}. With the
// 16x16x32 operand layout (lane l: tile row l % 16, k-chunk l / 16) these are tile rows 0-7 at
// chunk c with rows 8-15 at chunk c ^ 1, which the plain swizzle chunk ^ (row & 7) keeps apart
// (kind 0; the bank-conflict counter reads 0). A global_load_lds instruction always writes 64
// lanes x 16 bytes contiguously, so the swizzle is applied on the global-address side: each lane
// fetches the chunk that belongs at the LDS position it will be written to.
//
// Workgroup ids are remapped so that the 32 workgroups resident on one XCD (ids congruent mod 8)
// at any time are 32 consecutive tiles of the walk, a compact GROUP_M x 8 block of tiles that
// shares operand panels in that XCD's L2.
#pragma once
#include <type_traits>

#include "dppo_internal.h"

namespace dppo {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char lds_char;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NUM_XCD = 8, CU_PER_XCD = 32;   // MI355X: 8 XCDs of 32 compute units, one L2 each

struct TileCtx {
    int M, N;          // logical output size
    int tm, tn;        // tile coordinates
    int m0, n0;        // first row / column of this wavefront's sub-tile
    int bm0, bn0;      // first row / column of the workgroup tile
    int wave_m, wave_n, lane, tid;
    int item;          // work item of the launch (= tile when the launch does not split K)
    char* smem;
};

// 16x16x32 MFMA register layout: operand lane l holds row (A) or column (B) l % 16 and the 8
// k-values 8 * (l / 16) .. + 7; accumulator lane l holds column l % 16 and the 4 rows acc_row(l, j).
constexpr int MB = 16;    // rows / columns of an MFMA block
constexpr int MK = 32;    // k-values of one MFMA
__device__ __forceinline__ int acc_row(int lane, int j) { return 4 * (lane >> 4) + j; }
__device__ __forceinline__ int acc_col(int lane) { return lane & 15; }

#define DPPO_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define DPPO_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

// Waits until at most VM of this wavefront's global->LDS loads are outstanding and all its LDS
// reads have returned, then joins the workgroup barrier. Raw s_barrier: a __syncthreads() fence
// would also drain every outstanding load of the slices still in flight.
template <int VM>
__device__ __forceinline__ void wait_loads_then_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM) : "memory");
}

// Transposing LDS read: within each group of 16 lanes, lane i receives element i % 4 of the 8-byte
// rows addressed by lanes i / 4, 4 + i / 4, 8 + i / 4 and 12 + i / 4. The __restrict__ parameter
// gives the access an alias scope of its own; without one the compiler assumes that the read may
// alias the direct-to-LDS loads in flight and drains them all (vmcnt(0)) before every such read.
// The ordering against those loads is enforced by wait_loads_then_barrier.
__device__ __forceinline__ s16x4 lds_read_tr16(const lds_char* __restrict__ p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

// XOR term of the LDS swizzle: logical 16-byte chunk kc of tile row `row` lives at physical chunk
// kc ^ swz(row). Kinds 0..2: (row >> kind) & (CPR - 1) (kind 0 is the conflict-free choice for
// BK = 64, kind 2 for BK = 32); kind 3: (row & 7) ^ ((row >> 3) & 1).
template <int CPR, int SWZ> __device__ __forceinline__ int swz(int row) {
    if (SWZ == 3) return ((row & 7) ^ ((row >> 3) & 1)) & (CPR - 1);
    return (row >> SWZ) & (CPR - 1);
}

// BM x BN x BK tile, WGM x WGN wavefronts, STAGES slices of B and STAGES + AX slices of A in
// flight (A is the operand that streams from HBM in all three GEMMs of the path, B the one that
// stays cache-resident; with 2 + 1 stages of 32 KB A slices and 2 of B the 160 KB of LDS are used
// up and the A loads get two slice times to land instead of one), swizzle kind SWZ; SPREAD must be
// 1 (all loads of a slice are issued in the k-step that frees their buffers); GROUP_M tile rows
// form one band of the tile walk.
template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int STAGES_, int SWZ_, int SPREAD_, int GROUP_M_, int AX_ = 0>
struct PipeCfg {
    static constexpr int SA = STAGES_ + AX_, SB = STAGES_;   // ring depths of the A and B slices
    static constexpr int GROUP_M = GROUP_M_;   // tile rows per band of the tile walk
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, STAGES = STAGES_;
    static constexpr int SWZ = SWZ_, SPREAD = SPREAD_;
    static constexpr int NW = WGM * WGN, NT = NW * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MI = WTM / MB, NI = WTN / MB;
    static constexpr int KK = BK / MK;
    static constexpr int ROWB = BK * 2;
    static constexpr int CPR = BK / 8;
    static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    static constexpr int B_RING = SA * A_BYTES;               // LDS offset of the B ring
    static constexpr int LDS_BYTES = SA * A_BYTES + SB * B_BYTES;
    static constexpr int A_LD = A_BYTES / 1024 / NW;
    static constexpr int B_LD = B_BYTES / 1024 / NW;
    static constexpr int LPS = A_LD + B_LD;
    static_assert(SPREAD == 1, "spread");
    static_assert(AX_ == 0 || AX_ == 1, "extra A stages");
    static_assert(BK == 32 || BK == 64 || BK == 128, "BK");
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile vs wavefront count");
    static_assert(SA * LPS <= 63, "vmcnt range");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(NI >= 3 && NI <= MI && LPS <= MI, "read and load slots of a k-step");
};

// Layout of the A operand (template parameter AM):
//   A_ROWS      A is [M, K], K contiguous, lda = row pitch;
//   A_BLK_ROWS  A is a row-major [M, lda] matrix stored in blocks of BLK_R x BLK_C elements,
//               element (r, c) at blk_offset(r, c, lda); the GEMM's rows are the matrix rows and
//               K runs along its columns (the dH GEMM reads the gradient-logits chunk this way);
//   A_BLK_KM    the same blocked matrix, but the GEMM's K runs along the matrix ROWS and its M
//               along the columns (the dW GEMM: no transposed copy of the chunk is ever made).
// In the blocked layout a BK x BM slice of a tile (A_BLK_KM) is one contiguous 32 KB run and the
// rows of a BM x BK slice (A_BLK_ROWS) stay inside four such runs; a plain [K, M] matrix read tile
// by tile touches BK widely separated rows per slice and new pages at every slice.
// A_BLK_KM: the slice sits in LDS as BK rows of BM elements and the MFMA operand (8 consecutive k
// for one m per lane) is gathered by two transposing reads. The 16-byte chunks of a k-row are
// XOR-swizzled by 4 * (k & 3) + 2 * ((k >> 3) & 1) so that the 4 k-rows x 32 bytes a group of 16
// lanes touches, and the two groups of a half-wave (same columns, k-rows 8 apart), fall into
// different banks.
enum { A_ROWS = 0, A_BLK_ROWS = 1, A_BLK_KM = 2 };
// Layouts of the B operand ([N, K], K contiguous in both):
//   B_ROWS  row-major, ldb = row pitch;
//   B_BLK   in blocks of BN rows x BK columns, block (tile column tn, slice kt) at ((tn * K / BK) + kt) * BN * BK,
//           row-major inside: the slice a tile loads is one contiguous 32 KB run instead of BN pieces of
//           128 bytes a row pitch apart (with pitches of 64 KB to 300 KB that costs 5 % of the dH main loop's
//           cycles and 2.5 % of dW's). N is padded to whole blocks; ldb is not used.
enum { B_ROWS = 0, B_BLK = 1 };
constexpr int BLK_R = 64, BLK_C = 256;
__host__ __device__ __forceinline__ size_t blk_offset(int64_t r, int64_t c, int64_t ld) {
    return (size_t)(r / BLK_R) * BLK_R * ld + (size_t)(c / BLK_C) * (BLK_R * BLK_C) + (r % BLK_R) * BLK_C + c % BLK_C;
}

// Tile walk: tiles are numbered in bands of GROUP_M tile rows, column by column inside a band.
template <int GROUP_M>
__host__ __device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int& tm, int& tn) {
    // (one runtime division: this runs at the head of every workgroup, before its first load)
    const int band_sz = GROUP_M * tiles_n;
    const int band = tile / band_sz, in_band = tile - band * band_sz;
    const int first_m = band * GROUP_M;
    if (tiles_m - first_m >= GROUP_M) {          // a full band: GROUP_M is a compile-time constant
        tm = first_m + in_band % GROUP_M;
        tn = in_band / GROUP_M;
    } else {
        const int gm = tiles_m - first_m;
        tm = first_m + in_band % gm;
        tn = in_band / gm;
    }
}

// A launch covers gridDim.x work items: item i is part i % k_parts of tile tile0 + i / k_parts,
// and part p of a tile computes the k-slices [p KT / k_parts, (p + 1) KT / k_parts) of it
// (k_parts = 1: whole tiles).
enum { WG_ROUNDS = 0, WG_RANGES = 1 };
template <class Cfg, class Epi, int AM = A_ROWS, int MAP = WG_ROUNDS, int BL = B_ROWS>
__global__ __launch_bounds__(Cfg::NT) void gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                          const uint16_t* __restrict__ B, int64_t ldb, int M,
                                                          int N, int K, int tiles_m, int tiles_n, int tile0,
                                                          int k_parts, Epi epi, unsigned long long* phase) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // phase (benchmark aid, normally NULL): 4 counters that every workgroup adds to: shader cycles from
    // its start to the first slice in LDS, in the main loop, in the epilogue, and 1.
    unsigned long long pt0 = 0, pt1 = 0, pt2 = 0;
    if (phase) pt0 = clock64();
    constexpr bool A_KM = AM == A_BLK_KM;
    constexpr int MI = Cfg::MI, NI = Cfg::NI, KK = Cfg::KK, LPS = Cfg::LPS;
    constexpr int ROWB = Cfg::ROWB, CPR = Cfg::CPR;

    // Workgroup id -> work item. Ids congruent mod NUM_XCD run on the same XCD, in id order, one
    // per compute unit at a time, and all tiles of a launch take about the same time: the j-th
    // "round" of an XCD is its workgroups 32 j .. 32 j + 31.
    // WG_ROUNDS: round j of XCD x gets the 32 consecutive items of group 8 j + x, so that what
    // shares that XCD's L2 at any time is one compact block of the tile walk.
    // WG_RANGES: every XCD gets one contiguous range of items (round boundaries then fall
    // anywhere in the bands, but consecutive rounds of an XCD are neighbours in the walk).
    // The vocabulary GEMM (bands of 4 x 126 tiles) uses rounds: 38 against 45 GB of L2 misses per
    // launch. dH and dW (one-row bands of 10 tiles) use ranges.
    const int total = gridDim.x;
    int logical = blockIdx.x;
    {
        const int bid = blockIdx.x;
        const int xcd = bid % NUM_XCD, idx = bid / NUM_XCD;
        if (MAP == WG_ROUNDS) {
            constexpr int ROUND = NUM_XCD * CU_PER_XCD;
            if (bid < total / ROUND * ROUND)         // the last, partial round keeps the identity
                logical = ((idx / CU_PER_XCD) * NUM_XCD + xcd) * CU_PER_XCD + idx % CU_PER_XCD;
        } else {
            const int per = total / NUM_XCD, rem = total % NUM_XCD;
            logical = (xcd < rem) ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
        }
    }
    int tm, tn;
    int kt_lo = 0, kt_hi = K / Cfg::BK, item_tile = logical;
    if (k_parts != 1) {                          // whole tiles (the common case) skip these divisions
        item_tile = logical / k_parts;
        const int k_part = logical - item_tile * k_parts;
        kt_lo = (int)((int64_t)k_part * (K / Cfg::BK) / k_parts);
        kt_hi = (int)((int64_t)(k_part + 1) * (K / Cfg::BK) / k_parts);
    }
    tile_coords<Cfg::GROUP_M>(tile0 + item_tile, tiles_m, tiles_n, tm, tn);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS targets in SGPRs
    const int wave_m = wave % Cfg::WGM, wave_n = wave / Cfg::WGM;
    const int bm0 = tm * Cfg::BM, bn0 = tn * Cfg::BN;

    // one pointer per load (A loads first, then B loads)
    const uint16_t* pl[LPS];
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
        const bool isA = i < Cfg::A_LD;
        const int ii = isA ? i : i - Cfg::A_LD;
        const int ci = (ii * Cfg::NW + wave) * 64 + lane;
        if (A_KM && isA) {
            static_assert(!A_KM || (BLK_R % Cfg::BK == 0 && Cfg::BM == BLK_C), "a slice stays inside one block");
            constexpr int CPR_A = Cfg::BM / 8;
            const int krow = ci / CPR_A, pc = ci % CPR_A;
            const int mc = pc ^ (4 * (krow & 3) + 2 * ((krow >> 3) & 1));
            pl[i] = A + blk_offset(krow, bm0 + mc * 8, lda);
            continue;
        }
        const int row = ci / CPR, pc = ci % CPR;
        const int kc = pc ^ swz<CPR, Cfg::SWZ>(row);
        if (BL == B_BLK && !isA) {
            pl[i] = B + ((size_t)tn * (K / Cfg::BK) * Cfg::BN + row) * Cfg::BK + kc * 8;
            continue;
        }
        int r = (isA ? bm0 : bn0) + row;
        const int lim = isA ? M : N;
        r = r < lim ? r : lim - 1;
        if (AM == A_BLK_ROWS && isA) {
            static_assert(AM != A_BLK_ROWS || BLK_C % Cfg::BK == 0, "a slice stays inside one block column");
            pl[i] = A + blk_offset(r, kc * 8, lda);
            continue;
        }
        pl[i] = (isA ? A : B) + (size_t)r * (isA ? lda : ldb) + kc * 8;
    }
    // Issues load i of slice kt: i < B_LD is a B load into B-ring buffer bufb, the others are A loads
    // into A-ring buffer bufa. B goes first, so that at the next barrier "all but the newest A_LD
    // loads" means: this slice's B loads have landed, its A loads (due one slice later) may not have.
    auto issue_load = [&](int bufa, int bufb, int kt_rel, int i) {
        const int64_t kt = kt_lo + kt_rel;
        const size_t koff = (size_t)kt * Cfg::BK;
        const size_t koff_a = A_KM ? blk_offset(kt * Cfg::BK, 0, lda)
                              : AM == A_BLK_ROWS ? blk_offset(0, kt * Cfg::BK, lda) : koff;
        const bool isA = i >= Cfg::B_LD;
        const int ii = isA ? i - Cfg::B_LD : i;
        char* dst = smem + (isA ? bufa * Cfg::A_BYTES : Cfg::B_RING + bufb * Cfg::B_BYTES) + (ii * Cfg::NW + wave) * 1024;
        const uint16_t* src = isA ? pl[ii] + koff_a : pl[Cfg::A_LD + ii] + (BL == B_BLK ? koff * Cfg::BN : koff);
        __builtin_amdgcn_global_load_lds(DPPO_GPTR(src), DPPO_LPTR(dst), 16, 0, 0);
    };

    // Operand registers. Block mi of A is needed by NI consecutive MFMAs of a k-step and is dead
    // after them, so the blocks 0 .. MI-2 are single-buffered: the next k-step's block is read into
    // the same registers right after its last use. The last block would then be read at the very
    // end of the k-step, so it alone has two register sets and is read first. B blocks are needed
    // throughout a k-step and are double-buffered.
    const int frag_row = lane & 15, frag_q = lane >> 4;
    const int sw = swz<CPR, Cfg::SWZ>(frag_row);
    const int a_base = (wave_m * Cfg::WTM + frag_row) * ROWB;
    const int b_base = (wave_n * Cfg::WTN + frag_row) * ROWB;
    bf16x8 af[MI + 1], bfr[2][NI];
    auto a_slot = [](int mi, int parity) { return mi == MI - 1 ? MI - 1 + parity : mi; };
    // A_BLK_KM: byte offset, inside the A slice, of this lane's 8-byte source row for block mi at
    // k-step 0 (first of the two transposing reads; the second is 4 k-rows further on). A group of
    // 16 lanes reads 4 k-rows x 32 bytes; groups 0,1 (2,3) of a half-wave differ in bit 3 of k.
    constexpr int ROWB_A = Cfg::BM * 2;
    int a_km[MI];
    if (A_KM) {
        static_assert(!A_KM || (Cfg::WTM % 128 == 0 && MI <= 8), "swizzle of the [K, M] slice");
        const int s16 = lane & 15;
        const int xl = 2 * (s16 >> 2) + (frag_q & 1);            // (swizzle term of the k-row) / 2
        const int lane_off = (8 * frag_q + (s16 >> 2)) * ROWB_A + wave_m * (Cfg::WTM * 2) + ((s16 & 3) >> 1) * 16 +
                             (s16 & 1) * 8;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a_km[mi] = lane_off + 32 * (mi ^ xl);
    }
    auto read_a = [&](int slot, const char* st, int kk, int mi) {
        if (A_KM) {
            const lds_char* p = (const lds_char*)(st + a_km[mi] + kk * MK * ROWB_A);
            const s16x4 lo = lds_read_tr16(p);
            const s16x4 hi = lds_read_tr16(p + 4 * ROWB_A);
            const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            af[slot] = __builtin_bit_cast(bf16x8, v);
        } else {
            const int kc_off = ((kk * 4 + frag_q) ^ sw) << 4;
            af[slot] = *reinterpret_cast<const bf16x8*>(st + a_base + mi * MB * ROWB + kc_off);
        }
    };
    auto read_b = [&](int set, const char* st, int kk, int ni) {
        const int kc_off = ((kk * 4 + frag_q) ^ sw) << 4;
        bfr[set][ni] = *reinterpret_cast<const bf16x8*>(st + b_base + ni * MB * ROWB + kc_off);
    };

    f32x4 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[mi][ni][j] = 0.0f;

    const int KT = kt_hi - kt_lo;
    constexpr int SA = Cfg::SA, SB = Cfg::SB, A_LD = Cfg::A_LD, B_LD = Cfg::B_LD;
    // Slice kt has its A part in A-ring buffer kt % SA and its B part in B-ring buffer kt % SB. The
    // barrier at the last k-step of slice kt releases both buffers of slice kt, and the loads
    // [B of slice kt+SB, A of slice kt+SA] are issued behind it, in that order. Prologue: the same
    // groups for the virtual slices -SA .. -1.
#pragma unroll
    for (int j = -SA; j < 0; ++j) {
        if (j + SB >= 0 && j + SB < KT) {
#pragma unroll
            for (int i = 0; i < B_LD; ++i) issue_load(0, (j + SB) % SB, j + SB, i);
        }
        if (j + SA < KT) {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) issue_load((j + SA) % SA, 0, j + SA, B_LD + i);
        }
    }
    // loads issued behind B of slice 0: A of slices 1 .. SA-1 and B of slices 1 .. SB-1
    if (KT >= SA) wait_loads_then_barrier<(SA - 1) * A_LD + (SB - 1) * B_LD>();
    else wait_loads_then_barrier<0>();
    if (phase) pt1 = clock64();
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) read_a(a_slot(mi, 0), smem, 0, mi);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) read_b(0, smem + Cfg::B_RING, 0, ni);

    // One slice = KK k-steps. STEADY iterations (1 <= kt, kt + SA < KT) have every condition
    // resolved at compile time, so the whole slice is straight-line code. PAR = parity of the
    // slice's first k-step (which B register set it computes from); always 0 when KK is even.
    // At the barrier of slice kt the data of slice kt+1 must have landed; behind its B part were
    // issued (in steady state) SB-2 whole groups and, if the A ring is deeper, the A part of the
    // group that brought it.
    constexpr int STEADY_PENDING = (SB - 2) * LPS + (SA > SB ? A_LD : 0);
    int bufa = 0, bufb = 0;
    auto slice = [&](int kt, auto steady_tag, auto parity_tag) __attribute__((always_inline)) {
        constexpr bool STEADY = decltype(steady_tag)::value;
        constexpr int PAR = decltype(parity_tag)::value;
        const int nbufa = (bufa + 1 == SA) ? 0 : bufa + 1;
        const int nbufb = (bufb + 1 == SB) ? 0 : bufb + 1;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int cur = (kk + PAR) & 1, nxt = cur ^ 1;
            // Issue priority: low in the k-steps that run up to the barrier, high in the one behind it.
            // The two wavefronts of a SIMD drift apart (the older one wins every issue slot, reaches the
            // barrier first and idles there while the other one's memory instructions stall with nobody
            // to fill the matrix pipe); with the lagging wavefront preferred they reach the barrier
            // together (barrier wait of the leading wavefront 35 % -> 23 % of the loop, 3 % fewer cycles).
            if (kk == 0) __builtin_amdgcn_s_setprio(0);
            bool loads_a = false, loads_b = false, reads_here = false;
            int read_bufa = 0, read_bufb = 0, read_kk = 0;
            if (kk == KK - 1) {
                if (STEADY || kt + 1 < KT) {
                    if (STEADY) wait_loads_then_barrier<STEADY_PENDING>();
                    else wait_loads_then_barrier<0>();
                    __builtin_amdgcn_s_setprio(2);
                    loads_b = STEADY || kt + SB < KT;
                    loads_a = STEADY || kt + SA < KT;
                    read_bufa = nbufa; read_bufb = nbufb; read_kk = 0; reads_here = true;
                }
            } else {
                read_bufa = bufa; read_bufb = bufb; read_kk = kk + 1; reads_here = true;
            }
            {
                // Instruction order of a k-step, pinned by scheduling barriers (left to itself the
                // compiler sinks the reads next to their use and exposes the LDS latency). MFMA q
                // works on block (q / NI, q % NI); behind it, in the row of A block mi = q / NI:
                //   first MFMA of the step: the next step's last A block (into its spare registers),
                //   2nd MFMA of rows 0 .. NI-1: the next step's B block mi,
                //   3rd MFMA of rows 0 .. LPS-1: one global load (B loads first),
                //   last MFMA of rows 0 .. MI-2: the next step's A block mi, over the one just used.
                const char* rsa = smem + read_bufa * Cfg::A_BYTES;
                const char* rsb = smem + Cfg::B_RING + read_bufb * Cfg::B_BYTES;
#pragma unroll
                for (int q = 0; q < MI * NI; ++q) {
                    const int mi = q / NI, ni = q % NI;
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[a_slot(mi, cur)], bfr[cur][ni], acc[mi][ni], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (reads_here) {
                        if (q == 0) read_a(a_slot(MI - 1, nxt), rsa, read_kk, MI - 1);
                        if (ni == 1 && mi < NI) read_b(nxt, rsb, read_kk, mi);
                        if (ni == NI - 1 && mi < MI - 1) read_a(mi, rsa, read_kk, mi);
                    }
                    if (ni == 2 && mi < LPS) {
                        if (mi < B_LD) { if (loads_b) issue_load(bufa, bufb, kt + SB, mi); }
                        else if (loads_a) issue_load(bufa, bufb, kt + SA, mi);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        bufa = nbufa; bufb = nbufb;
    };
    typedef std::integral_constant<int, 0> P0;
    typedef std::integral_constant<int, 1> P1;
    int kt = 0;
    if (KT > 0) { slice(0, std::false_type{}, P0{}); kt = 1; }
    if (KK & 1) {
        // odd KK: the register-set parity alternates from slice to slice; kt stays odd here, so
        // slices go in pairs of parity (1, 0)
        for (; kt + 1 + SA < KT; kt += 2) { slice(kt, std::true_type{}, P1{}); slice(kt + 1, std::true_type{}, P0{}); }
        for (; kt + 1 < KT; kt += 2) { slice(kt, std::false_type{}, P1{}); slice(kt + 1, std::false_type{}, P0{}); }
        if (kt < KT) slice(kt, std::false_type{}, P1{});
    } else {
        for (; kt + SA < KT; ++kt) slice(kt, std::true_type{}, P0{});
        for (; kt < KT; ++kt) slice(kt, std::false_type{}, P0{});
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_s_setprio(0);
    if (phase) pt2 = clock64();

    TileCtx c;
    c.M = M; c.N = N; c.tm = tm; c.tn = tn;
    c.bm0 = bm0; c.bn0 = bn0;
    c.m0 = bm0 + wave_m * Cfg::WTM; c.n0 = bn0 + wave_n * Cfg::WTN;
    c.wave_m = wave_m; c.wave_n = wave_n; c.lane = lane; c.tid = tid; c.item = logical; c.smem = smem;
    epi.template run<Cfg>(acc, c);
    if (phase && tid == 0) {
        const unsigned long long pt3 = clock64();
        atomicAdd(phase + 0, pt1 - pt0);
        atomicAdd(phase + 1, pt2 - pt1);
        atomicAdd(phase + 2, pt3 - pt2);
        atomicAdd(phase + 3, 1ull);
    }
}

// ---------------------------------------------------------------------------------------
// Epilogues
// ---------------------------------------------------------------------------------------
// Store of the accumulators. KIND 0 (dW): float output, overwrite or accumulate. KIND 1 (dH):
// bf16 output, optional row scatter through row_map.
// dW is a read-modify-write of 256 KB per tile; straight from the accumulator layout it would be
// 4-byte accesses in 64-byte runs, so the tile goes through LDS (free after the main loop) in two
// halves of BM/2 rows = the rows of one wavefront row, and leaves as 16-byte accesses that cover
// whole 1 KB output rows. The sums are the same numbers in the same order.
template <int KIND>
struct EpiStore {
    float* Cf; uint16_t* Cb; int64_t ldc; int accumulate; const int32_t* row_map; int64_t row_base;
    const float* row_scale;   // KIND 1: output row m is multiplied by row_scale[m] if not NULL
    float* partial;           // if not NULL, work item i stores its whole BM x BN fp32 tile, row-major, at
                              // partial + i * BM * BN instead (launches that split K; summed up by a second kernel)

    template <class Cfg>
    __device__ __forceinline__ void run(f32x4 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
        if (KIND == 0) {
            static_assert(KIND != 0 || Cfg::WGM == 2, "one half of the tile per wavefront row");
            typedef float f32x4v __attribute__((ext_vector_type(4)));
            constexpr int PITCH = Cfg::BN * 4 + 16;           // bytes per staged row
            constexpr int HALF = Cfg::BM / 2;
            constexpr int VPR = Cfg::BN / 4;                   // float4 per row
            constexpr int RPP = Cfg::NT / VPR;                 // rows per pass
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (c.wave_m == h) {
#pragma unroll
                    for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < Cfg::NI; ++ni)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int r = mi * MB + acc_row(c.lane, j);
                                const int col = c.wave_n * Cfg::WTN + ni * MB + acc_col(c.lane);
                                *reinterpret_cast<float*>(c.smem + r * PITCH + col * 4) = acc[mi][ni][j];
                            }
                }
                __syncthreads();
                const int cv = c.tid % VPR;
                const int col = c.bn0 + cv * 4;
#pragma unroll 4
                for (int r = c.tid / VPR; r < HALF; r += RPP) {
                    const int row = c.bm0 + h * HALF + r;
                    if (partial) {
                        *reinterpret_cast<f32x4v*>(partial + (size_t)c.item * (Cfg::BM * Cfg::BN) +
                                                   (size_t)(h * HALF + r) * Cfg::BN + cv * 4) =
                            *reinterpret_cast<const f32x4v*>(c.smem + r * PITCH + cv * 16);
                    } else if (row < c.M && col < c.N) {
                        f32x4v v = *reinterpret_cast<const f32x4v*>(c.smem + r * PITCH + cv * 16);
                        f32x4v* dst = reinterpret_cast<f32x4v*>(Cf + (size_t)row * ldc + col);
                        if (accumulate) v += *dst;
                        *dst = v;
                    }
                }
                __syncthreads();
            }
            return;
        }
        if (partial) {       // K-split launch: the raw fp32 tile, row-major, to this work item's slot
            float* dst = partial + (size_t)c.item * (Cfg::BM * Cfg::BN);
#pragma unroll
            for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = c.wave_m * Cfg::WTM + mi * MB + acc_row(c.lane, j);
#pragma unroll
                    for (int ni = 0; ni < Cfg::NI; ++ni)
                        dst[(size_t)r * Cfg::BN + c.wave_n * Cfg::WTN + ni * MB + acc_col(c.lane)] = acc[mi][ni][j];
                }
            return;
        }
#pragma unroll
        for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = c.m0 + mi * MB + acc_row(c.lane, j);
                if (row >= c.M) continue;
                const int64_t orow = row_map ? (int64_t)row_map[row_base + row] : (int64_t)row;
                const float rs = row_scale ? row_scale[row] : 1.0f;
#pragma unroll
                for (int ni = 0; ni < Cfg::NI; ++ni) {
                    const int col = c.n0 + ni * MB + acc_col(c.lane);
                    if (col >= c.N) continue;
                    const __bf16 h = (__bf16)(acc[mi][ni][j] * rs);
                    Cb[(size_t)orow * ldc + col] = __builtin_bit_cast(uint16_t, h);
                }
            }
    }

    // KIND 0 needs N and ldc to be multiples of 4 and C 16-byte aligned (checked by the launcher).
    template <class Cfg>
    static constexpr int lds_bytes() { return KIND == 0 ? (Cfg::BM / 2) * (Cfg::BN * 4 + 16) : 0; }
};
typedef EpiStore<0> EpiStoreDW;
typedef EpiStore<1> EpiStoreDH;

constexpr float LOG2E = 1.4426950408889634f;

// Stores the BN x BM tile staged in LDS as [token][vocabulary row] (pitch ZPITCH bytes, 2-byte
// elements) to the blocked chunk dst (pitch ld elements): 16-byte vectors, 32 lanes per 512-byte row.
template <class Cfg>
__device__ __forceinline__ void store_staged_row(const TileCtx& c, uint16_t* dst, int64_t ld, int r, int ch) {
    constexpr int ZPITCH = Cfg::BM * 2 + 16;
    const u32x4 val = *reinterpret_cast<const u32x4*>(c.smem + r * ZPITCH + ch * 16);
    // streaming store: the chunk (10 GB) is not read again before it has left every cache, and a
    // regular store would evict the operand panels the other tiles of the group share in L2
    __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(dst + blk_offset(c.bn0 + r, c.bm0 + ch * 8, ld)));
}

// Rows = vocabulary entries, columns = tokens: per-(row tile, token) running max and sum of
// exponentials, nothing else leaves the tile.
struct EpiLogits {
    float2* part; int64_t n_cp;    // part[tile_m * n_cp + token]

    template <class Cfg>
    __device__ __forceinline__ void run(f32x4 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
        constexpr int MI = Cfg::MI, NI = Cfg::NI;
        const float NEG_INF = -__builtin_inff();
        float2* red = reinterpret_cast<float2*>(c.smem);   // (max, sum) pairs of the WGM wavefronts that share a token
        // running max over this wavefront's vocabulary rows, per token column: in-lane over the
        // blocks, then across the four lane groups that hold the column's other rows.
        // Only the last row of tiles has vocabulary rows beyond M; every other tile takes the
        // branch that is compiled without the row masks.
        float mx[NI], sm[NI];
        auto reduce = [&](auto full_tag) __attribute__((always_inline)) {
            constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                float m = NEG_INF;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int row = c.m0 + mi * MB + acc_row(c.lane, j);
                        const float v = (FULL || row < c.M) ? acc[mi][ni][j] : NEG_INF;
                        m = fmaxf(m, v);
                    }
                m = fmaxf(m, __shfl_xor(m, 16, 64));
                m = fmaxf(m, __shfl_xor(m, 32, 64));
                mx[ni] = m;
                const float mref = (m == NEG_INF) ? 0.0f : m;
                float s = 0.0f;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int row = c.m0 + mi * MB + acc_row(c.lane, j);
                        const float ex = __builtin_amdgcn_exp2f((acc[mi][ni][j] - mref) * LOG2E);
                        s += (FULL || row < c.M) ? ex : 0.0f;
                    }
                sm[ni] = s;
            }
        };
        if (c.bm0 + Cfg::BM <= c.M) reduce(std::true_type{});
        else reduce(std::false_type{});
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            sm[ni] += __shfl_xor(sm[ni], 16, 64);
            sm[ni] += __shfl_xor(sm[ni], 32, 64);
        }
        if (c.lane < MB) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                red[c.wave_m * Cfg::BN + c.wave_n * Cfg::WTN + ni * MB + c.lane] = make_float2(mx[ni], sm[ni]);
        }
        __syncthreads();
        for (int t = c.tid; t < Cfg::BN; t += Cfg::NT) {
            float m = NEG_INF;
#pragma unroll
            for (int w = 0; w < Cfg::WGM; ++w) m = fmaxf(m, red[w * Cfg::BN + t].x);
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < Cfg::WGM; ++w) {
                const float2 r = red[w * Cfg::BN + t];
                s += (r.x == NEG_INF) ? 0.0f : r.y * __builtin_amdgcn_exp2f((r.x - m) * LOG2E);
            }
            const int64_t tok = c.bn0 + t;
            if (tok < n_cp) part[(int64_t)c.tm * n_cp + tok] = make_float2(m, s);
        }
    }

    template <class Cfg>
    static constexpr int lds_bytes() { return Cfg::WGM * Cfg::BN * 8; }
};

// Rows = vocabulary entries, columns = tokens. What the backward pass needs of the logits is the
// softmax, and exp(z - lse) cannot be formed before the whole row has been seen; but bf16 has the
// exponent range of fp32, so the tile stores E[n, v] = exp(z[n, v] - b[n]) against any per-token
// reference b[n] that is within the exponent range of lse[n]. The softmax gradient is then a row
// scaling of E, c[n] (1[v = y] - p[n, v]) = s[n] (E[n, v] - 1[v = y] exp(lse[n] - b[n])) with
// s[n] = -c[n] exp(b[n] - lse[n]), which the two backward GEMMs apply on their small operands, and
// the stored chunk is never read and rewritten by an elementwise pass. E goes to the blocked
// chunk as bf16 (0 for the vocabulary padding). part[tile][token] = (max z, sum exp(z - b)) over
// the tile's rows: the sums of all tiles share the reference and just add up; the max gives the
// caller a safe reference for redoing the rows whose reference was too far off.
struct EpiLogitsExp {
    float2* part; int64_t n_cp;
    const float* bref;
    uint16_t* E; int64_t lde;      // [n_cp, lde] in BLK_R x BLK_C blocks (blk_offset)

    template <class Cfg>
    __device__ __forceinline__ void run(f32x4 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
        constexpr int MI = Cfg::MI, NI = Cfg::NI;
        static_assert(Cfg::BM == BLK_C && Cfg::BN % BLK_R == 0, "tile = whole blocks");
        const float NEG_INF = -__builtin_inff();
        // LDS (free after the main loop's closing barrier): the tile's E as bf16, laid out
        // [token][vocabulary row] so that it leaves as 16-byte stores that fill the tile's four
        // 32 KB blocks of the chunk, then the per-wavefront (max, sum) pairs.
        constexpr int ZPITCH = Cfg::BM * 2 + 16;      // bytes per token row; +16 staggers the banks
        float2* red = reinterpret_cast<float2*>(c.smem + Cfg::BN * ZPITCH);
        float mx[NI], sm[NI], bl[NI];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int64_t col = c.bn0 + c.wave_n * Cfg::WTN + ni * MB + acc_col(c.lane);
            bl[ni] = (col < n_cp ? bref[col] : 0.0f) * LOG2E;
            mx[ni] = NEG_INF;
            sm[ni] = 0.0f;
        }
        // The stores of a tile leave slowly (every compute unit reaches its epilogue at about the
        // same time, and together they saturate the write path), so the work is cut into the NI
        // token blocks of a wavefront column: while the 16-byte stores of block q - 1 drain (32 lanes
        // x 16 bytes = one 512-byte token row piece, two rows per instruction), the exponentials of
        // block q are computed and staged.
        constexpr int CH = Cfg::BM / 8;                     // 16-byte chunks per row
        constexpr int RPP = Cfg::NT / CH;                   // token rows per store pass
        constexpr int PART_ROWS = Cfg::BN / NI;             // token rows of one part
        constexpr int PASSES = PART_ROWS / RPP;             // store passes per part
        static_assert(PART_ROWS % RPP == 0 && MI % PASSES == 0, "block rows per store pass");
        constexpr int GPP = MI / PASSES;
        const int ch = c.tid % CH;
        auto body = [&](auto full_tag) __attribute__((always_inline)) {
            constexpr bool FULL = decltype(full_tag)::value;
            auto stage = [&](int ni, int mi) __attribute__((always_inline)) {
                const int tok = c.wave_n * Cfg::WTN + ni * MB + acc_col(c.lane);
                const int vloc = c.wave_m * Cfg::WTM + mi * MB + acc_row(c.lane, 0);
                bf16x4 h;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float z = acc[mi][ni][q];
                    const bool ok = FULL || (c.bm0 + vloc + q < c.M);
                    float e = __builtin_amdgcn_exp2f(__builtin_fmaf(z, LOG2E, -bl[ni]));
                    e = ok ? e : 0.0f;
                    mx[ni] = fmaxf(mx[ni], ok ? z : NEG_INF);
                    sm[ni] += e;
                    const __bf16 b = (__bf16)e;   // scalar copy: reading h[q] back right after writing it miscompiles
                    h[q] = b;
                }
                *reinterpret_cast<bf16x4*>(c.smem + tok * ZPITCH + vloc * 2) = h;
            };
            auto store_pass = [&](int part, int it) __attribute__((always_inline)) {
                const int idx = it * RPP + c.tid / CH;                    // row among the part's rows
                const int r = (idx / MB) * Cfg::WTN + part * MB + idx % MB;
                store_staged_row<Cfg>(c, E, lde, r, ch);
            };
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) stage(0, mi);
            __syncthreads();
#pragma unroll
            for (int part = 1; part < NI; ++part) {
#pragma unroll
                for (int it = 0; it < PASSES; ++it) {
                    store_pass(part - 1, it);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int e = 0; e < GPP; ++e) stage(part, it * GPP + e);
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();
            }
#pragma unroll
            for (int it = 0; it < PASSES; ++it) store_pass(NI - 1, it);
        };
        if (c.bm0 + Cfg::BM <= c.M) body(std::true_type{});
        else body(std::false_type{});
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            mx[ni] = fmaxf(mx[ni], __shfl_xor(mx[ni], 16, 64));
            mx[ni] = fmaxf(mx[ni], __shfl_xor(mx[ni], 32, 64));
            sm[ni] += __shfl_xor(sm[ni], 16, 64);
            sm[ni] += __shfl_xor(sm[ni], 32, 64);
        }
        if (c.lane < MB) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                red[c.wave_m * Cfg::BN + c.wave_n * Cfg::WTN + ni * MB + c.lane] = make_float2(mx[ni], sm[ni]);
        }
        __syncthreads();
        for (int t = c.tid; t < Cfg::BN; t += Cfg::NT) {
            float m = NEG_INF, s = 0.0f;
#pragma unroll
            for (int w = 0; w < Cfg::WGM; ++w) {
                const float2 r = red[w * Cfg::BN + t];
                m = fmaxf(m, r.x);
                s += r.y;
            }
            const int64_t tok = c.bn0 + t;
            if (tok < n_cp) part[(int64_t)c.tm * n_cp + tok] = make_float2(m, s);
        }
    }

    template <class Cfg>
    static constexpr int lds_bytes() { return Cfg::BN * (Cfg::BM * 2 + 16) + Cfg::WGM * Cfg::BN * 8; }
};

// Rows = vocabulary entries, columns = tokens: softmax-gradient entries straight from the logits,
// staged through LDS as [token][vocabulary row] and stored to the blocked chunk like the logits.
struct EpiLogitsGrad {
    const int32_t* y; const float* lse; const float* cvec;
    uint16_t* G; int64_t ldg; int64_t n_cp; int V;

    template <class Cfg>
    __device__ __forceinline__ void run(f32x4 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
        static_assert(Cfg::BM == BLK_C && Cfg::BN % BLK_R == 0, "tile = whole blocks");
        constexpr int ZPITCH = Cfg::BM * 2 + 16;
#pragma unroll
        for (int ni = 0; ni < Cfg::NI; ++ni) {
            const int tok = c.wave_n * Cfg::WTN + ni * MB + acc_col(c.lane);
            const int64_t col = c.bn0 + tok;
            const bool col_ok = col < n_cp;
            const int yt = col_ok ? y[col] : -1;
            const float l = col_ok ? lse[col] : 0.0f;
            const float cn = col_ok ? cvec[col] : 0.0f;
#pragma unroll
            for (int mi = 0; mi < Cfg::MI; ++mi) {
                const int vloc = c.wave_m * Cfg::WTM + mi * MB + acc_row(c.lane, 0);
                bf16x4 h;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int v = c.bm0 + vloc + q;
                    const float p = __builtin_amdgcn_exp2f((acc[mi][ni][q] - l) * LOG2E);
                    float gv = cn * ((v == yt ? 1.0f : 0.0f) - p);
                    gv = v < V ? gv : 0.0f;
                    const __bf16 b = (__bf16)gv;   // scalar copy: reading h[q] back right after writing it miscompiles
                    h[q] = b;
                }
                *reinterpret_cast<bf16x4*>(c.smem + tok * ZPITCH + vloc * 2) = h;
            }
        }
        __syncthreads();
        constexpr int CH = Cfg::BM / 8;
        constexpr int ROWS_PER_PASS = Cfg::NT / CH;
        const int ch = c.tid % CH;
#pragma unroll 4
        for (int r = c.tid / CH; r < Cfg::BN; r += ROWS_PER_PASS) store_staged_row<Cfg>(c, G, ldg, r, ch);
    }

    template <class Cfg>
    static constexpr int lds_bytes() { return Cfg::BN * (Cfg::BM * 2 + 16); }
};

}  // namespace mfma
}  // namespace dppo
