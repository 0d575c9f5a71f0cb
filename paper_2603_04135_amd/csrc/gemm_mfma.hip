// Instantiations and host launchers of the bf16 MFMA GEMM kernels (see gemm_mfma_kernel.h).
#include "gemm_mfma_kernel.h"

namespace dppo {
namespace {
using namespace mfma;

// 256x256x64 tile, 2x4 wavefronts (128x64 each), 3 A slices and 2 B slices in flight (all 160 KB of
// LDS), all loads of a slice issued in the k-step that frees its buffers, bands of 4 tile rows. The
// blocked chunk layout (64 x 256 element blocks) is tied to this tile.
typedef PipeCfg<256, 256, 64, 2, 4, 2, 0, 1, 4, 1> CfgBig;

// Dynamic LDS of a kernel: the operand slices, or the epilogue's staging area if that is larger.
template <class Cfg, class Epi>
constexpr int lds_request() {
    constexpr int e = Epi::template lds_bytes<Cfg>();
    static_assert(e <= 160 * 1024, "epilogue LDS");
    return Cfg::LDS_BYTES > e ? Cfg::LDS_BYTES : e;
}

template <class Cfg, int AM = A_ROWS, class Epi>
void launch(const void* A, int64_t lda, const void* B, int64_t ldb, int M, int N, int K, const Epi& epi,
            hipStream_t st) {
    const int tiles_m = (int)ceil_div(M, Cfg::BM), tiles_n = (int)ceil_div(N, Cfg::BN);
    gemm_nt_kernel<Cfg, Epi, AM><<<dim3(tiles_m * tiles_n), dim3(Cfg::NT), lds_request<Cfg, Epi>(), st>>>(
        reinterpret_cast<const uint16_t*>(A), lda, reinterpret_cast<const uint16_t*>(B), ldb, M, N, K, tiles_m,
        tiles_n, epi);
}

template <class Cfg, class Epi, int AM = A_ROWS>
hipError_t allow_lds() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<Cfg, Epi, AM>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_request<Cfg, Epi>());
}

}  // namespace

int mfma_setup() {
    static int status = [] {
        hipError_t e = allow_lds<CfgBig, EpiStoreDW, A_BLK_KM>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiStoreDH, A_BLK_ROWS>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogits>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogitsExp>();
        if (e == hipSuccess) e = allow_lds<CfgBig, EpiLogitsGrad>();
        if (e != hipSuccess) return fail(DPPO_ERR_DEVICE, "hipFuncSetAttribute(dynamic LDS): %s", hipGetErrorString(e));
        return (int)DPPO_OK;
    }();
    return status;
}

int32_t mfma_logits_row_tiles(int32_t V) { return (int32_t)ceil_div(V, CfgBig::BM); }
int32_t mfma_vocab_tile() { return CfgBig::BM; }

void launch_mfma_logits(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                        hipStream_t st) {
    EpiLogits e{part, n_cp};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
}

int launch_mfma_logits_exp(const void* W, int32_t V, int32_t D, const void* Hc, int32_t n_cp, float2* part,
                           const float* bref, void* E, int64_t lde, int32_t Vp, hipStream_t st) {
    // the epilogue stores whole tiles: the caller pads the row pitch to whole vocabulary tiles
    if (Vp % CfgBig::BM != 0 || lde != Vp || Vp < V)
        return fail(DPPO_ERR_UNSUPPORTED, "chunk buffer not padded to whole vocabulary tiles (Vp %d, pitch %lld)", Vp,
                    (long long)lde);
    EpiLogitsExp e{part, n_cp, bref, reinterpret_cast<uint16_t*>(E), lde};
    launch<CfgBig>(W, D, Hc, D, V, n_cp, D, e, st);
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

void launch_mfma_dh(const void* G, int32_t Vp, const void* WT, int32_t n_c, int32_t D, const float* row_scale,
                    const StoreSpec& out, hipStream_t st) {
    EpiStoreDH e{nullptr, reinterpret_cast<uint16_t*>(out.C), out.ldc, 0, out.row_map, out.row_base, row_scale};
    launch<CfgBig, A_BLK_ROWS>(G, Vp, WT, Vp, n_c, D, Vp, e, st);
}

void launch_mfma_dw(const void* G, int32_t Vp, const void* HcT, int32_t n_cp, int32_t V, int32_t D,
                    const StoreSpec& out, hipStream_t st) {
    EpiStoreDW e{reinterpret_cast<float*>(out.C), nullptr, out.ldc, out.accumulate, nullptr, 0, nullptr};
    launch<CfgBig, A_BLK_KM>(G, Vp, HcT, n_cp, V, D, n_cp, e, st);
}

}  // namespace dppo
