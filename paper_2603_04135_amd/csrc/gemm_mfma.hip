// bf16 MFMA GEMM for gfx950, C[M,N] = A[M,K] * B[N,K]^T with both operands K-contiguous,
// and the epilogues of the LM-head path fused onto its accumulators:
//   * vocabulary GEMM (rows = vocabulary entries, columns = tokens): running max / sum-exp per
//     token over the tile's vocabulary rows, so full logits never reach HBM; optionally the
//     chunk's logits as fp16, or directly the softmax-gradient entries in bf16;
//   * plain stores (fp32 / bf16, overwrite or accumulate, optional row scatter) for dH and dW.
// One workgroup owns a BM x BN output tile and streams K in steps of 64 through LDS
// (double-buffered, XOR-swizzled 16-byte chunks so the ds_read_b128 of an MFMA operand are
// bank-conflict free); each wavefront owns a (BM/WGM) x (BN/WGN) sub-tile made of 32x32x16
// MFMA blocks. Workgroup ids are remapped so that the workgroups resident on one XCD (ids
// congruent mod 8) cover a compact block of tiles and share operand panels in that XCD's L2.
#include "dppo_internal.h"

namespace dppo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;            // K step (bf16 elements): one 128-byte LDS row per tile row
constexpr int ROW_BYTES = BK * 2;
constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;        // tile rows per band of the tile walk

template <int BM_, int BN_, int WGM_, int WGN_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;   // 16-byte chunks per thread
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(NT % 64 == 0 && (NT / 8) % 8 == 0, "thread count");
    static_assert(BM % (NT / 8) == 0 && BN % (NT / 8) == 0, "tile rows per load pass");
};

struct TileCtx {
    int M, N;          // logical output size
    int tm, tn;        // tile coordinates
    int m0, n0;        // first row / column of this wavefront's sub-tile
    int bm0, bn0;      // first row / column of the workgroup tile
    int wave_m, wave_n, lane, tid;
    char* smem;
};

// Row of accumulator element j (0..15) of a 32x32 MFMA block, relative to the block.
__device__ __forceinline__ int acc_row(int lane, int j) { return 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3); }

template <class Cfg, class Epi>
__global__ __launch_bounds__(Cfg::NT) void gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                          const uint16_t* __restrict__ B, int64_t ldb, int M,
                                                          int N, int K, int tiles_m, int tiles_n, Epi epi) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int MI = Cfg::MI, NI = Cfg::NI;

    // ---- workgroup id -> tile, XCD-aware ------------------------------------------------
    const int total = tiles_m * tiles_n;
    int logical;
    {
        const int bid = blockIdx.x;
        const int xcd = bid % NUM_XCD, idx = bid / NUM_XCD;
        const int per = total / NUM_XCD, rem = total % NUM_XCD;
        logical = (xcd < rem) ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
    }
    int tm, tn;
    {
        const int band_sz = GROUP_M * tiles_n;
        const int band = logical / band_sz, in_band = logical % band_sz;
        const int first_m = band * GROUP_M;
        const int gm = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
        tm = first_m + in_band % gm;
        tn = in_band / gm;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % Cfg::WGM, wave_n = wave / Cfg::WGM;
    const int bm0 = tm * Cfg::BM, bn0 = tn * Cfg::BN;

    // ---- global -> LDS staging assignment: thread owns 16-byte chunk (row, kc) of each pass
    const int ld_row = tid >> 3, ld_kc = tid & 7;
    const int ld_lds = ld_row * ROW_BYTES + ((ld_kc ^ (ld_row & 7)) << 4);
    const uint16_t* pa[Cfg::A_CH];
    const uint16_t* pb[Cfg::B_CH];
#pragma unroll
    for (int i = 0; i < Cfg::A_CH; ++i) {
        int r = bm0 + ld_row + i * (Cfg::NT / 8);
        r = r < M ? r : M - 1;
        pa[i] = A + (size_t)r * lda + ld_kc * 8;
    }
#pragma unroll
    for (int i = 0; i < Cfg::B_CH; ++i) {
        int r = bn0 + ld_row + i * (Cfg::NT / 8);
        r = r < N ? r : N - 1;
        pb[i] = B + (size_t)r * ldb + ld_kc * 8;
    }

    // ---- LDS -> MFMA operand addressing ------------------------------------------------
    const int frag_row = lane & 31, frag_half = lane >> 5, sw = lane & 7;
    const int a_base = (wave_m * Cfg::WTM + frag_row) * ROW_BYTES;
    const int b_base = Cfg::A_BYTES + (wave_n * Cfg::WTN + frag_row) * ROW_BYTES;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[mi][ni][j] = 0.0f;

    u32x4 ra[Cfg::A_CH], rb[Cfg::B_CH];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < Cfg::A_CH; ++i) ra[i] = *reinterpret_cast<const u32x4*>(pa[i] + (size_t)kt * BK);
#pragma unroll
        for (int i = 0; i < Cfg::B_CH; ++i) rb[i] = *reinterpret_cast<const u32x4*>(pb[i] + (size_t)kt * BK);
    };
    auto store_lds = [&](int stage) {
        char* base = smem + stage * Cfg::STAGE_BYTES + ld_lds;
#pragma unroll
        for (int i = 0; i < Cfg::A_CH; ++i)
            *reinterpret_cast<u32x4*>(base + i * (Cfg::NT / 8) * ROW_BYTES) = ra[i];
#pragma unroll
        for (int i = 0; i < Cfg::B_CH; ++i)
            *reinterpret_cast<u32x4*>(base + Cfg::A_BYTES + i * (Cfg::NT / 8) * ROW_BYTES) = rb[i];
    };

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_global(kt + 1);
        const char* st = smem + (kt & 1) * Cfg::STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kc_off = ((kk * 2 + frag_half) ^ sw) << 4;
            bf16x8 af[MI], bf[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[mi] = *reinterpret_cast<const bf16x8*>(st + a_base + mi * 32 * ROW_BYTES + kc_off);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bf[ni] = *reinterpret_cast<const bf16x8*>(st + b_base + ni * 32 * ROW_BYTES + kc_off);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bf[ni], acc[mi][ni], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    TileCtx c;
    c.M = M; c.N = N; c.tm = tm; c.tn = tn;
    c.bm0 = bm0; c.bn0 = bn0;
    c.m0 = bm0 + wave_m * Cfg::WTM; c.n0 = bn0 + wave_n * Cfg::WTN;
    c.wave_m = wave_m; c.wave_n = wave_n; c.lane = lane; c.tid = tid; c.smem = smem;
    epi.template run<Cfg>(acc, c);
}

// ---------------------------------------------------------------------------------------
// Epilogues
// ---------------------------------------------------------------------------------------
// Plain store of the accumulators. KIND 0 (dW): float output, overwrite or accumulate.
// KIND 1 (dH): bf16 output, optional row scatter through row_map.
template <int KIND>
struct EpiStore {
    float* Cf; uint16_t* Cb; int64_t ldc; int accumulate; const int32_t* row_map; int64_t row_base;

    template <class Cfg>
    __device__ __forceinline__ void run(f32x16 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
#pragma unroll
        for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int row = c.m0 + mi * 32 + acc_row(c.lane, j);
                if (row >= c.M) continue;
                const int64_t orow = (KIND == 1 && row_map) ? (int64_t)row_map[row_base + row] : (int64_t)row;
#pragma unroll
                for (int ni = 0; ni < Cfg::NI; ++ni) {
                    const int col = c.n0 + ni * 32 + (c.lane & 31);
                    if (col >= c.N) continue;
                    const float v = acc[mi][ni][j];
                    const size_t idx = (size_t)orow * ldc + col;
                    if (KIND == 1) {
                        const __bf16 h = (__bf16)v;
                        Cb[idx] = __builtin_bit_cast(uint16_t, h);
                    } else {
                        Cf[idx] = accumulate ? Cf[idx] + v : v;
                    }
                }
            }
    }
};
typedef EpiStore<0> EpiStoreDW;
typedef EpiStore<1> EpiStoreDH;

constexpr float LOG2E = 1.4426950408889634f;

// Rows = vocabulary entries, columns = tokens.
template <bool STORE_Z>
struct EpiLogits {
    float2* part; int64_t n_cp;    // part[tile_m * n_cp + token]
    _Float16* Z16; int64_t ldz; int Vp;

    template <class Cfg>
    __device__ __forceinline__ void run(f32x16 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
        constexpr int MI = Cfg::MI, NI = Cfg::NI;
        const float NEG_INF = -__builtin_inff();
        float mx[NI], sm[NI];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            float m = NEG_INF;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int row = c.m0 + mi * 32 + acc_row(c.lane, j);
                    const float v = row < c.M ? acc[mi][ni][j] : NEG_INF;
                    m = fmaxf(m, v);
                }
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            const float mref = (m == NEG_INF) ? 0.0f : m;
            float s = 0.0f;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int row = c.m0 + mi * 32 + acc_row(c.lane, j);
                    const float e = __builtin_amdgcn_exp2f((acc[mi][ni][j] - mref) * LOG2E);
                    s += row < c.M ? e : 0.0f;
                }
            s += __shfl_xor(s, 32, 64);
            mx[ni] = m; sm[ni] = s;
        }
        if (STORE_Z) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int64_t col = c.n0 + ni * 32 + (c.lane & 31);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int v0 = c.m0 + mi * 32 + 8 * g + 4 * (c.lane >> 5);
                        if (v0 < Vp) {
                            f16x4 h;
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                float z = acc[mi][ni][4 * g + q];
                                z = fminf(fmaxf(z, -65504.0f), 65504.0f);
                                h[q] = (_Float16)z;
                            }
                            *reinterpret_cast<f16x4*>(Z16 + col * ldz + v0) = h;
                        }
                    }
            }
        }
        // combine the WGM wavefronts that cover the same tokens
        __syncthreads();
        float2* red = reinterpret_cast<float2*>(c.smem);
        if (c.lane < 32) {
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                red[c.wave_m * Cfg::BN + c.wave_n * Cfg::WTN + ni * 32 + c.lane] = make_float2(mx[ni], sm[ni]);
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
};

// Rows = vocabulary entries, columns = tokens: softmax-gradient entries straight from the logits.
struct EpiLogitsGrad {
    const int32_t* y; const float* lse; const float* cvec;
    uint16_t* G; uint16_t* GT; int64_t ldg; int64_t n_cp; int V, Vp;

    template <class Cfg>
    __device__ __forceinline__ void run(f32x16 (&acc)[Cfg::MI][Cfg::NI], const TileCtx& c) const {
#pragma unroll
        for (int ni = 0; ni < Cfg::NI; ++ni) {
            const int64_t col = c.n0 + ni * 32 + (c.lane & 31);
            const bool col_ok = col < n_cp;
            const int yt = col_ok ? y[col] : -1;
            const float l = col_ok ? lse[col] : 0.0f;
            const float cn = col_ok ? cvec[col] : 0.0f;
#pragma unroll
            for (int mi = 0; mi < Cfg::MI; ++mi)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int v0 = c.m0 + mi * 32 + 8 * g + 4 * (c.lane >> 5);
                    if (v0 < Vp && col_ok) {
                        bf16x4 h;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int v = v0 + q;
                            const float p = __builtin_amdgcn_exp2f((acc[mi][ni][4 * g + q] - l) * LOG2E);
                            float gv = cn * ((v == yt ? 1.0f : 0.0f) - p);
                            gv = v < V ? gv : 0.0f;
                            const __bf16 b = (__bf16)gv;   // scalar copy: reading h[q] back right after writing it miscompiles
                            h[q] = b;
                            GT[(int64_t)v * n_cp + col] = __builtin_bit_cast(uint16_t, b);
                        }
                        *reinterpret_cast<bf16x4*>(G + col * ldg + v0) = h;
                    }
                }
        }
    }
};

typedef TileCfg<256, 256, 2, 2> CfgBig;

template <class Cfg, class Epi>
void launch(const void* A, int64_t lda, const void* B, int64_t ldb, int M, int N, int K, const Epi& epi,
            hipStream_t st) {
    const int tiles_m = (int)ceil_div(M, Cfg::BM), tiles_n = (int)ceil_div(N, Cfg::BN);
    gemm_nt_kernel<Cfg, Epi><<<dim3(tiles_m * tiles_n), dim3(Cfg::NT), Cfg::LDS_BYTES, st>>>(
        reinterpret_cast<const uint16_t*>(A), lda, reinterpret_cast<const uint16_t*>(B), ldb, M, N, K, tiles_m,
        tiles_n, epi);
}

template <class Cfg, class Epi>
hipError_t allow_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<Cfg, Epi>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
}

}  // namespace

int mfma_setup() {
    static int status = [] {
        hipError_t e = allow_lds<CfgBig, EpiStoreDW>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiStoreDH>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogits<true>>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogits<false>>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogitsGrad>();
        if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "hipFuncSetAttribute(dynamic LDS): %s", hipGetErrorString(e));
        return (int)DPPO_OK;
    }();
    return status;
}

int32_t mfma_logits_row_tiles(int32_t V) { return (int32_t)ceil_div(V, CfgBig::BM); }

void launch_mfma_logits(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                        void* Z16, int64_t ldz, int32_t Vp, hipStream_t st) {
    if (Z16) {
        EpiLogits<true> e{part, n_cp, reinterpret_cast<_Float16*>(Z16), ldz, Vp};
        launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
    } else {
        EpiLogits<false> e{part, n_cp, nullptr, 0, 0};
        launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
    }
}

void launch_mfma_logits_grad(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp,
                             const int32_t* y, const float* lse, const float* c, void* G, void* GT,
                             int64_t ldg, int32_t Vp, hipStream_t st) {
    EpiLogitsGrad e{y, lse, c, reinterpret_cast<uint16_t*>(G), reinterpret_cast<uint16_t*>(GT), ldg, n_cp, V, Vp};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
}

void launch_mfma_gemm(const void* A, int64_t lda, const void* B, int64_t ldb, int32_t M, int32_t N, int32_t K,
                      const StoreSpec& out, hipStream_t st) {
    if (out.out_bf16) {
        EpiStoreDH e{nullptr, reinterpret_cast<uint16_t*>(out.C), out.ldc, 0, out.row_map, out.row_base};
        launch<CfgBig>(A, lda, B, ldb, M, N, K, e, st);
    } else {
        EpiStoreDW e{reinterpret_cast<float*>(out.C), nullptr, out.ldc, out.accumulate, nullptr, 0};
        launch<CfgBig>(A, lda, B, ldb, M, N, K, e, st);
    }
}

}  // namespace dppo
