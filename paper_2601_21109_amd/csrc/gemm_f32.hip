// fp32 path of cwl_chunkwise_lora_linear: a plain LDS-tiled FMA GEMM over the concatenated
// reduction dimension (see linear_common.h).  Small shapes only matter here (the fp32
// configuration is a correctness case), so the kernel favours generality: any M, N, K.
#include "linear_common.h"

namespace cwl {
namespace {

constexpr int BM = 64, BN = 64, BK = 16;

template <int EPI>
__global__ void __launch_bounds__(256) gemm_f32_tn_kernel(GemmArgs a) {
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t bm = blockIdx.x / a.tiles_n, bn = blockIdx.x % a.tiles_n;
    const int64_t m0 = bm * BM, n0 = bn * BN;

    // loader role: one row of the tile, 4 consecutive k
    const int lrow = tid >> 2, lk = (tid & 3) * 4;
    const int64_t gm = m0 + lrow, gn = n0 + lrow;
    const bool m_ok = gm < a.M, n_ok = gn < a.N;
    const int64_t tok = m_ok ? (a.perm ? a.perm[gm] : gm) : 0;

    int32_t r_tile = 0;
    if (a.blk_r) r_tile = a.blk_r[m0 / kRankBlock];   // BM == kRankBlock

    float acc[4][4] = {};
    for (int part = 0; part < 2; ++part) {
        const float* Ap = static_cast<const float*>(part == 0 ? a.A1 : a.A2);
        const float* Bp = static_cast<const float*>(part == 0 ? a.B1 : a.B2);
        const int64_t lda = part == 0 ? a.lda1 : a.lda2;
        const int64_t ldb = part == 0 ? a.ldb1 : a.ldb2;
        const int64_t arow = part == 0 ? tok : gm;
        const int32_t Kp = part == 0 ? a.K1 : r_tile;
        for (int32_t k0 = 0; k0 < Kp; k0 += BK) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int32_t k = k0 + lk + i;
                As[lk + i][lrow] = (m_ok && k < Kp) ? Ap[arow * lda + k] : 0.0f;
                Bs[lk + i][lrow] = (n_ok && k < Kp) ? Bp[gn * ldb + k] : 0.0f;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < BK; ++k) {
                float av[4], bv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
            }
            __syncthreads();
        }
    }

    float* C = static_cast<float*>(a.C);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t g = m0 + ty * 4 + i;
        if (g >= a.M) continue;
        const int64_t t = a.perm ? a.perm[g] : g;
        if (EPI == EPI_GATE) {
            const TokMeta mt = a.meta[t];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + tx * 4 + j;
                if (n >= a.N) continue;
                const int64_t dir = a.gate_period > 0 ? n % a.gate_period : n;   // direction within its adapter
                const float gate = (dir < mt.r_prev ? mt.g_prev : 0.0f) + (dir < mt.r_cur ? mt.g_cur : 0.0f);
                C[g * a.ldc + n] = acc[i][j] * gate;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + tx * 4 + j;
                if (n < a.N) C[t * a.ldc + n] = acc[i][j];
            }
        }
    }
}

}  // namespace

cwl_status launch_gemm_f32(const GemmArgs& a_in, int epi, hipStream_t st) {
    GemmArgs a = a_in;
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t blocks = (int64_t)a.tiles_m * a.tiles_n;
    if (blocks <= 0) return CWL_OK;
    if (blocks >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    if (epi == EPI_GATE)
        gemm_f32_tn_kernel<EPI_GATE><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
    else
        gemm_f32_tn_kernel<EPI_STORE><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace cwl
