// fp32 GEMM C[M,N] = A[M,K] * B[N,K]^T for the float32 data type of the LM-head path.
// Any M, N, K; LDS-tiled FMA code (64x64 tile, 4x4 per thread). It serves the small fp32
// configuration and is not the tuned path (that is the bf16 MFMA kernel).
#include "dppo_internal.h"

namespace dppo {
namespace {

constexpr int PT = 64;   // tile edge
constexpr int PK = 16;   // K step

__global__ __launch_bounds__(256) void gemm_plain_kernel(const float* __restrict__ A, int64_t lda,
                                                         const float* __restrict__ B, int64_t ldb, int M, int N,
                                                         int K, float* Cf, uint16_t* Cb, int64_t ldc,
                                                         int accumulate, const int32_t* row_map,
                                                         int64_t row_base) {
    __shared__ float As[PK][PT + 4];
    __shared__ float Bs[PK][PT + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * PT, n0 = blockIdx.x * PT;
    const int tr = tid / 16, tc = tid % 16;   // 4x4 micro-tile: rows tr*4.., cols tc*4..
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += PK) {
        for (int e = tid; e < PT * PK; e += 256) {
            const int r = e / PK, k = e % PK;
            const int gm = m0 + r, gn = n0 + r, gk = k0 + k;
            As[k][r] = (gm < M && gk < K) ? A[(size_t)gm * lda + gk] : 0.0f;
            Bs[k][r] = (gn < N && gk < K) ? B[(size_t)gn * ldb + gk] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < PK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][tr * 4 + i]; b[i] = Bs[k][tc * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        const int row = m0 + tr * 4 + i;
        if (row >= M) continue;
        const int64_t orow = row_map ? (int64_t)row_map[row_base + row] : (int64_t)row;
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tc * 4 + j;
            if (col >= N) continue;
            const size_t idx = (size_t)orow * ldc + col;
            if (Cb) {
                __bf16 h = (__bf16)acc[i][j];
                Cb[idx] = __builtin_bit_cast(uint16_t, h);
            } else {
                Cf[idx] = accumulate ? Cf[idx] + acc[i][j] : acc[i][j];
            }
        }
    }
}

}  // namespace

void launch_gemm_plain_f32(const float* A, int64_t lda, const float* B, int64_t ldb, int32_t M, int32_t N,
                           int32_t K, const StoreSpec& out, hipStream_t st) {
    if (M <= 0 || N <= 0) return;
    dim3 grid((unsigned)ceil_div(N, PT), (unsigned)ceil_div(M, PT));
    gemm_plain_kernel<<<grid, 256, 0, st>>>(A, lda, B, ldb, M, N, K,
                                            out.out_bf16 ? nullptr : reinterpret_cast<float*>(out.C),
                                            out.out_bf16 ? reinterpret_cast<uint16_t*>(out.C) : nullptr, out.ldc,
                                            out.accumulate, out.row_map, out.row_base);
}

}  // namespace dppo
