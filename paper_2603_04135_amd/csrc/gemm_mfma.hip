// Instantiations and host launchers of the bf16 MFMA GEMM kernels (see gemm_mfma_kernel.h).
#include <atomic>
#include <mutex>

#include "gemm_mfma_kernel.h"

namespace dppo {
namespace {
using namespace mfma;

// 256x256x64 tile, 2x4 wavefronts (128x64 each), 3 A slices and 2 B slices in flight (all 160 KB of
// LDS), all loads of a slice issued in the k-step that frees its buffers. The blocked chunk layout
// (64 x 256 element blocks) is tied to this tile. The GEMMs differ only in the band height of the
// tile walk: 4 tile rows for the vocabulary GEMM (126 token tiles per row: 4 x 8 blocks per L2);
// 1 for dH and dW, whose rows have only D / 256 = 10 tiles: the A panels there are pieces of the
// 10 GB chunk that streams from HBM, and with one-row bands all 10 users of a panel are
// consecutive tiles and run in the same round (bands of 4 x 10 tiles straddle the rounds of 32:
// dH +1.6 %, dW +1.2 % in time); with such bands a contiguous range of rows per XCD (WG_RANGES)
// is as good (dW) or 0.9 % better (dH) than interleaved rounds.
typedef PipeCfg<256, 256, 64, 2, 4, 2, 0, 1, 4, 1> CfgBig;
typedef PipeCfg<256, 256, 64, 2, 4, 2, 0, 1, 1, 1> CfgGrad;
static_assert(CfgGrad::BN == GEMM_B_BLOCK_ROWS && CfgGrad::BK == GEMM_B_BLOCK_K, "blocked B operand = the tile's slices");

// Dynamic LDS of a kernel: the operand slices, or the epilogue's staging area if that is larger.
template <class Cfg, class Epi>
constexpr int lds_request() {
    constexpr int e = Epi::template lds_bytes<Cfg>();
    static_assert(e <= 160 * 1024, "epilogue LDS");
    return Cfg::LDS_BYTES > e ? Cfg::LDS_BYTES : e;
}

// Launches the tiles [tile0, tile0 + n_tiles) of the tile walk, each cut into k_parts work items
// along K; n_tiles < 0: all tiles.
// Tile-phase counters of the benchmark aid (NULL = off): 4 counters per GEMM stage, see gemm_nt_kernel.
std::atomic<unsigned long long*> g_phase_counters{nullptr};
enum { PHASE_LOGITS = 0, PHASE_DH = 1, PHASE_DW = 2 };

template <class Cfg, int AM = A_ROWS, int MAP = WG_ROUNDS, int BL = B_ROWS, class Epi>
void launch(const void* A, int64_t lda, const void* B, int64_t ldb, int M, int N, int K, const Epi& epi,
            hipStream_t st, int tile0 = 0, int n_tiles = -1, int k_parts = 1, int phase_stage = -1) {
    const int tiles_m = (int)ceil_div(M, Cfg::BM), tiles_n = (int)ceil_div(N, Cfg::BN);
    if (n_tiles < 0) n_tiles = tiles_m * tiles_n - tile0;
    if (n_tiles <= 0) return;
    unsigned long long* phase = phase_stage >= 0 && k_parts == 1 ? g_phase_counters.load() : nullptr;
    if (phase) phase += 4 * phase_stage;
    gemm_nt_kernel<Cfg, Epi, AM, MAP, BL><<<dim3(n_tiles * k_parts), dim3(Cfg::NT), lds_request<Cfg, Epi>(), st>>>(
        reinterpret_cast<const uint16_t*>(A), lda, reinterpret_cast<const uint16_t*>(B), ldb, M, N, K, tiles_m,
        tiles_n, tile0, k_parts, epi, phase);
}

// Sums the k_parts partial tiles of each of the n_tiles tiles from tile0 on, in part order, into
// C (overwrite or accumulate). One workgroup per 16 rows of a tile; N and ldc multiples of 4.
// With Cb != NULL the sums go out as bf16 instead: row m times row_scale[m] (if not NULL) to row
// row_map[row_base + m] (if not NULL) of Cb.
template <class Cfg>
__global__ __launch_bounds__(256) void sum_partial_tiles_kernel(const float* __restrict__ partial, int tile0,
                                                                int k_parts, int tiles_m, int tiles_n, float* C,
                                                                int64_t ldc, int M, int N, int accumulate,
                                                                uint16_t* Cb, const int32_t* __restrict__ row_map,
                                                                int64_t row_base, const float* __restrict__ row_scale) {
    typedef float f32x4v __attribute__((ext_vector_type(4)));
    constexpr int VPR = Cfg::BN / 4;
    int tm, tn;
    tile_coords<Cfg::GROUP_M>(tile0 + blockIdx.x, tiles_m, tiles_n, tm, tn);
    const float* src = partial + (size_t)blockIdx.x * k_parts * (Cfg::BM * Cfg::BN);
    for (int i = threadIdx.x; i < 16 * VPR; i += 256) {
        const int r = blockIdx.y * 16 + i / VPR, cv = i % VPR;
        const int row = tm * Cfg::BM + r, col = tn * Cfg::BN + cv * 4;
        if (row >= M || col >= N) continue;
        f32x4v v = *reinterpret_cast<const f32x4v*>(src + (size_t)r * Cfg::BN + cv * 4);
        for (int p = 1; p < k_parts; ++p)
            v += *reinterpret_cast<const f32x4v*>(src + (size_t)p * (Cfg::BM * Cfg::BN) + (size_t)r * Cfg::BN + cv * 4);
        if (Cb) {
            const float rs = row_scale ? row_scale[row] : 1.0f;
            const int64_t orow = row_map ? (int64_t)row_map[row_base + row] : (int64_t)row;
            const __bf16 b0 = (__bf16)(v[0] * rs), b1 = (__bf16)(v[1] * rs), b2 = (__bf16)(v[2] * rs), b3 = (__bf16)(v[3] * rs);
            const uint32_t lo = (uint32_t)__builtin_bit_cast(uint16_t, b0) | ((uint32_t)__builtin_bit_cast(uint16_t, b1) << 16);
            const uint32_t hi = (uint32_t)__builtin_bit_cast(uint16_t, b2) | ((uint32_t)__builtin_bit_cast(uint16_t, b3) << 16);
            *reinterpret_cast<uint2*>(Cb + (size_t)orow * ldc + col) = make_uint2(lo, hi);
            continue;
        }
        f32x4v* dst = reinterpret_cast<f32x4v*>(C + (size_t)row * ldc + col);
        if (accumulate) v += *dst;
        *dst = v;
    }
}

template <class Cfg, class Epi, int AM = A_ROWS, int MAP = WG_ROUNDS, int BL = B_ROWS>
hipError_t allow_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<Cfg, Epi, AM, MAP, BL>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_request<Cfg, Epi>());
}

}  // namespace

// Per-device state: the dynamic-LDS attribute of every GEMM kernel and the number of compute
// units, looked up once for each device a bfloat16 call runs on.
namespace {
constexpr int MAX_DEVICES = 64;
struct DeviceState { bool done = false; int status = DPPO_OK; int cus = 0; };
DeviceState g_dev[MAX_DEVICES];
std::mutex g_dev_mu;
}  // namespace

int mfma_setup(int* compute_units) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(DPPO_ERR_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lk(g_dev_mu);
    DeviceState& d = g_dev[dev];
    if (!d.done) {
        e = hipDeviceGetAttribute(&d.cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = allow_lds<CfgGrad, EpiStoreDW, A_BLK_KM, WG_RANGES, B_BLK>();
        if (e == hipSuccess) e = allow_lds<CfgGrad, EpiStoreDH, A_BLK_ROWS, WG_RANGES, B_BLK>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogits>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogitsExp>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogitsGrad>();
        d.status = e == hipSuccess ? (int)DPPO_OK
                                   : fail(DPPO_ERR_DEVICE, "device %d setup (dynamic LDS): %s", dev, hipGetErrorString(e));
        d.done = e == hipSuccess;    // a failed setup is tried again by the next call
        if (e != hipSuccess) return d.status;
    }
    if (compute_units) *compute_units = d.cus;
    return d.status;
}

void mfma_set_phase_counters(unsigned long long* counters) { g_phase_counters.store(counters); }

int32_t mfma_logits_row_tiles(int32_t V) { return (int32_t)ceil_div(V, CfgBig::BM); }
int32_t mfma_vocab_tile() { return CfgBig::BM; }

void launch_mfma_logits(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                        hipStream_t st) {
    EpiLogits e{part, n_cp};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st, 0, -1, 1, PHASE_LOGITS);
}

int launch_mfma_logits_exp(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                           const float* bref, void* E, int64_t lde, int32_t Vp, hipStream_t st) {
    // the epilogue stores whole tiles: the caller pads the row pitch to whole vocabulary tiles
    if (Vp % CfgBig::BM != 0 || lde != Vp || Vp < V)
        return fail(DPPO_ERR_UNSUPPORTED, "chunk buffer not padded to whole vocabulary tiles (Vp %d, pitch %lld)", Vp,
                    (long long)lde);
    EpiLogitsExp e{part, n_cp, bref, reinterpret_cast<uint16_t*>(E), lde};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st, 0, -1, 1, PHASE_LOGITS);
    return DPPO_OK;
}

int launch_mfma_logits_grad(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp,
                            const int32_t* y, const float* lse, const float* c, void* G, int64_t ldg,
                            int32_t Vp, hipStream_t st) {
    if (Vp % CfgBig::BM != 0 || ldg != Vp || Vp < V)
        return fail(DPPO_ERR_UNSUPPORTED, "gradient-logits buffer not padded to whole vocabulary tiles (Vp %d, pitch %lld)",
                    Vp, (long long)ldg);
    EpiLogitsGrad e{y, lse, c, reinterpret_cast<uint16_t*>(G), ldg, n_cp, V};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
    return DPPO_OK;
}

size_t mfma_dw_partial_bytes() { return (size_t)256 * CfgBig::BM * CfgBig::BN * 4; }

// One workgroup per compute unit at a time: the last round of tiles holds tiles % cus of them. If
// that is at most half the chip, those tiles are cut along K into as many parts as fill it (at
// most 8, at least 16 slices each), each part writes its partial tile to scratch, and a small
// kernel adds the parts up in order (the same sums in a different association; deterministic).
// Returns the number of parts (1 = no split) and the number of tail tiles.
static int tail_split(int cus, int tiles, int k_slices, const float* partial, int& tail) {
    tail = cus > 0 ? tiles % cus : 0;
    int parts = 1;
    if (partial && tail > 0 && 2 * tail <= cus) {
        parts = cus / tail;
        if (parts > 8) parts = 8;
        if (parts > k_slices / 16) parts = k_slices / 16;
        if ((size_t)tail * parts * CfgBig::BM * CfgBig::BN * 4 > mfma_dw_partial_bytes()) parts = 1;
    }
    return parts < 2 ? 1 : parts;
}

void launch_mfma_dh(int cus, const void* G, int32_t Vp, const void* WT, int32_t n_c, int32_t D, const float* row_scale,
                    const StoreSpec& out, float* partial, hipStream_t st) {
    EpiStoreDH e{nullptr, reinterpret_cast<uint16_t*>(out.C), out.ldc, 0, out.row_map, out.row_base, row_scale, nullptr};
    const int tiles_m = (int)ceil_div(n_c, CfgGrad::BM), tiles_n = (int)ceil_div(D, CfgGrad::BN);
    const int tiles = tiles_m * tiles_n;
    int tail;
    const int parts = tail_split(cus, tiles, Vp / CfgGrad::BK, partial, tail);
    if (parts == 1) {
        launch<CfgGrad, A_BLK_ROWS, WG_RANGES, B_BLK>(G, Vp, WT, 0, n_c, D, Vp, e, st, 0, -1, 1, PHASE_DH);
        return;
    }
    launch<CfgGrad, A_BLK_ROWS, WG_RANGES, B_BLK>(G, Vp, WT, 0, n_c, D, Vp, e, st, 0, tiles - tail, 1, PHASE_DH);
    EpiStoreDH ep = e;
    ep.partial = partial;
    launch<CfgGrad, A_BLK_ROWS, WG_RANGES, B_BLK>(G, Vp, WT, 0, n_c, D, Vp, ep, st, tiles - tail, tail, parts);
    sum_partial_tiles_kernel<CfgGrad><<<dim3(tail, CfgGrad::BM / 16), 256, 0, st>>>(
        partial, tiles - tail, parts, tiles_m, tiles_n, nullptr, out.ldc, n_c, D, 0, reinterpret_cast<uint16_t*>(out.C),
        out.row_map, out.row_base, row_scale);
}

void launch_mfma_dw(int cus, const void* G, int32_t Vp, const void* HcT, int32_t n_cp, int32_t V, int32_t D,
                    const StoreSpec& out, float* partial, hipStream_t st) {
    EpiStoreDW e{reinterpret_cast<float*>(out.C), nullptr, out.ldc, out.accumulate, nullptr, 0, nullptr, nullptr};
    const int tiles_m = (int)ceil_div(V, CfgGrad::BM), tiles_n = (int)ceil_div(D, CfgGrad::BN);
    const int tiles = tiles_m * tiles_n;
    int tail;
    const int parts = tail_split(cus, tiles, n_cp / CfgGrad::BK, partial, tail);
    if (parts == 1) {
        launch<CfgGrad, A_BLK_KM, WG_RANGES, B_BLK>(G, Vp, HcT, 0, V, D, n_cp, e, st, 0, -1, 1, PHASE_DW);
        return;
    }
    launch<CfgGrad, A_BLK_KM, WG_RANGES, B_BLK>(G, Vp, HcT, 0, V, D, n_cp, e, st, 0, tiles - tail, 1, PHASE_DW);
    EpiStoreDW ep = e;
    ep.partial = partial;
    launch<CfgGrad, A_BLK_KM, WG_RANGES, B_BLK>(G, Vp, HcT, 0, V, D, n_cp, ep, st, tiles - tail, tail, parts);
    sum_partial_tiles_kernel<CfgGrad><<<dim3(tail, CfgGrad::BM / 16), 256, 0, st>>>(
        partial, tiles - tail, parts, tiles_m, tiles_n, reinterpret_cast<float*>(out.C), out.ldc, V, D, out.accumulate,
        nullptr, nullptr, 0, nullptr);
}

// Register-only loop of the GEMMs' MFMA instruction (8 wavefronts per compute unit, 32 independent
// accumulator blocks each, operands never leave the registers): the rate the matrix pipes sustain
// when nothing has to be loaded, which is the ceiling the GEMMs are priced against. With random operand
// values the chip's power limit lowers the clock, so the ceiling depends on the data.
namespace {
__device__ __forceinline__ mfma::bf16x8 probe_operand(unsigned seed, int random_values) {
    mfma::bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        unsigned h = (seed * 8u + (unsigned)i) * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        const float f = random_values ? (float)((int)(h % 2001u) - 1000) * 0.001f : 1.0f;
        v[i] = (__bf16)f;
    }
    return v;
}
__global__ __launch_bounds__(512) void mfma_rate_kernel(float* out, int iters, int random_values) {
    mfma::bf16x8 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = probe_operand(threadIdx.x * 7u + (unsigned)i + blockIdx.x * 1000u, random_values);
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = probe_operand(threadIdx.x * 13u + (unsigned)i + 77u, random_values);
    mfma::f32x4 acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = mfma::f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 32; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[q / 4], b[q % 4], acc[q], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (threadIdx.x == 0) out[blockIdx.x] = s;      // keeps the loop alive; one float per workgroup
}
}  // namespace

double launch_mfma_rate_probe(int cus, int iters, int random_values, float* out, hipStream_t st) {
    mfma_rate_kernel<<<cus, 512, 0, st>>>(out, iters, random_values);
    return (double)cus * 8.0 * (double)iters * 32.0 * 16384.0;   // 8 wavefronts x 32 MFMAs x 2 x 16 x 16 x 32 flop
}

}  // namespace dppo
