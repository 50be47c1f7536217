// cwl_build_ladder: the rank ladder of a trained adapter by one SVD of its update dW = A B (Sec. III-C
// of arxiv 2601.21109: the ladder is obtained once, offline, and a rung slices its first r directions).
// gfx950 only.  include/cwl.h states what is computed; this is how.
//
// dW is d_in x d_out but has rank <= r <= 256, so the SVD is taken through r x r matrices, in fp64:
//   1. Gram matrices G_A = A^T A and G_B = B B^T (whole chip: one 32 x 32 tile of G over one slab of
//      the samples per workgroup, the slabs added in a fixed order afterwards);
//   2. one workgroup: eigen-decompositions G_A = V_A L_A V_A^T, G_B = V_B L_B V_B^T, which give
//      A = Q_A (L_A^1/2 V_A^T) and B = (V_B L_B^1/2) Q_B^T with orthonormal Q_A = A V_A L_A^-1/2 and
//      Q_B^T = L_B^-1/2 V_B^T B; the core M = L_A^1/2 V_A^T V_B L_B^1/2; its SVD M = U S V^T, so that
//      dW = (Q_A U) S (Q_B V)^T; directions sorted by S; the two r x r maps
//           T_A = V_A L_A^-1/2 U S^1/2          T_B = S^1/2 V^T L_B^-1/2 V_B^T
//      (inverse square roots of eigenvalues below 1e-13 of the largest, and singular values below
//      1e-12 of the largest, count as zero: those directions carry nothing);
//   3. A' = A T_A and B' = T_B B (whole chip).
// All three decompositions use one routine, the one-sided Jacobi method (Hestenes): plane rotations
// from the right make the columns of X orthogonal, X V = Y; column norms of Y are the singular values
// (for a symmetric positive semi-definite X: the eigenvalues, and V the eigenvectors).  The r / 2
// disjoint column pairs of a round-robin round are rotated at once, a few threads per pair.  Up to
// r = 96 the two matrices of a decomposition are worked on in LDS; larger ones (up to 512 KiB each)
// stay in the workspace and are served from L2.  This is set-up work that runs once per adapter.
#include "common.h"

namespace cwl {
namespace {

constexpr int kCoreThreads = 1024;
constexpr int kMaxSweeps = 40;
constexpr double kRotTol = 1e-13;      // columns count as orthogonal below this cosine
constexpr double kEigTol = 1e-13;      // eigenvalues of a Gram matrix below this fraction of the largest: zero
constexpr double kSigTol = 1e-12;      // singular values below this fraction of the largest: zero

struct LadderWs {
    double *GA, *VA, *GB, *VB, *M, *VM, *TA, *TB;    // r x r each; G*, V*, M column-major, T* [k][i]
    double *PA, *PB;                                  // [slabs] partial Gram matrices, one per slab of samples
    double *lamA, *lamB, *sig;                        // [r]
    int32_t* perm;                                    // [r] column of M's SVD that has rank i
    int32_t slabs;
};

constexpr int kGramTile = 32, kGramSamples = 64;

// slabs of samples a Gram matrix is summed over: enough workgroups for the chip, at most 32
int32_t gram_slabs(int32_t r) {
    const int32_t tiles = (r + kGramTile - 1) / kGramTile;
    int32_t slabs = 256 / (tiles * tiles);
    return slabs < 1 ? 1 : (slabs > 32 ? 32 : slabs);
}

size_t ladder_ws_layout(int32_t r, void* base, LadderWs* ws) {
    const size_t mat = align_up(sizeof(double) * (size_t)r * (size_t)r, 256);
    const size_t vec = align_up(sizeof(double) * (size_t)r, 256);
    const int32_t slabs = gram_slabs(r);
    if (ws) {
        char* b = static_cast<char*>(base);
        double** mats[8] = {&ws->GA, &ws->VA, &ws->GB, &ws->VB, &ws->M, &ws->VM, &ws->TA, &ws->TB};
        for (int i = 0; i < 8; ++i) *mats[i] = reinterpret_cast<double*>(b + mat * i);
        ws->PA = reinterpret_cast<double*>(b + mat * 8);
        ws->PB = reinterpret_cast<double*>(b + mat * (8 + slabs));
        char* v = b + mat * (8 + 2 * (size_t)slabs);
        ws->lamA = reinterpret_cast<double*>(v);
        ws->lamB = reinterpret_cast<double*>(v + vec);
        ws->sig = reinterpret_cast<double*>(v + vec * 2);
        ws->perm = reinterpret_cast<int32_t*>(v + vec * 3);
        ws->slabs = slabs;
    }
    return mat * (8 + 2 * (size_t)slabs) + vec * 4;
}

__device__ __forceinline__ float load_elem(const void* p, int64_t idx, int bf16) {
    if (bf16) return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[idx]);
    return static_cast<const float*>(p)[idx];
}

__device__ __forceinline__ void store_elem(void* p, int64_t idx, float v, int bf16) {
    if (bf16) {
        uint32_t u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) u |= 0x00400000u;        // NaN stays NaN
        else u += 0x7fffu + ((u >> 16) & 1u);                          // nearest, ties to even
        static_cast<uint16_t*>(p)[idx] = (uint16_t)(u >> 16);
    } else {
        static_cast<float*>(p)[idx] = v;
    }
}

// ---- 1. Gram matrix over samples: G[i][j] = sum_s X(s, i) X(s, j), X(s, c) = X[s*ss + c*cs] ----
// A: sample = row (ss = lda, cs = 1); B: sample = column (ss = 1, cs = ldb).  blockIdx.z takes one slab
// of the samples and writes its own partial matrix; the core kernel adds the slabs in a fixed order.
__global__ void __launch_bounds__(256)
gram_kernel(const void* __restrict__ X, int bf16, int64_t n_all, int64_t ss, int64_t cs, int32_t r,
            double* __restrict__ P /*[slabs] column-major r x r*/) {
    const int64_t per = ((n_all + gridDim.z - 1) / gridDim.z + kGramSamples - 1) / kGramSamples * kGramSamples;
    const int64_t s_begin = (int64_t)blockIdx.z * per;
    const int64_t n_samples = s_begin + per < n_all ? s_begin + per : n_all;
    double* G = P + (size_t)blockIdx.z * r * r;
    __shared__ float sI[kGramSamples][kGramTile + 1];
    __shared__ float sJ[kGramSamples][kGramTile + 1];
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kGramTile, j0 = blockIdx.y * kGramTile;
    const int ti = (tid & 15) * 2, tj = (tid >> 4) * 2;
    double acc[2][2] = {{0, 0}, {0, 0}};
    const bool comp_fast = cs == 1;
    for (int64_t s0 = s_begin; s0 < n_samples; s0 += kGramSamples) {
        for (int e = tid; e < kGramSamples * kGramTile; e += 256) {
            const int c = comp_fast ? (e % kGramTile) : (e / kGramSamples);
            const int s = comp_fast ? (e / kGramTile) : (e % kGramSamples);
            const int64_t row = s0 + s;
            float vi = 0.0f, vj = 0.0f;
            if (row < n_samples) {
                if (i0 + c < r) vi = load_elem(X, row * ss + (int64_t)(i0 + c) * cs, bf16);
                if (j0 + c < r) vj = load_elem(X, row * ss + (int64_t)(j0 + c) * cs, bf16);
            }
            sI[s][c] = vi;
            sJ[s][c] = vj;
        }
        __syncthreads();
#pragma unroll 8
        for (int s = 0; s < kGramSamples; ++s) {
            const double a0 = sI[s][ti], a1 = sI[s][ti + 1], b0 = sJ[s][tj], b1 = sJ[s][tj + 1];
            acc[0][0] += a0 * b0;
            acc[0][1] += a0 * b1;
            acc[1][0] += a1 * b0;
            acc[1][1] += a1 * b1;
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
            if (i0 + ti + a < r && j0 + tj + b < r) G[(size_t)(j0 + tj + b) * r + (i0 + ti + a)] = acc[a][b];
}

// ---- 2. the r x r work, one workgroup ----

// One-sided Jacobi: on return the columns of X (column-major n x n) are mutually orthogonal,
// X_out = X_in V.  Every thread of the workgroup must call it.
__device__ void jacobi_sweeps(double* __restrict__ X, double* __restrict__ V, int32_t n, int* flag /*LDS*/);

// The matrices are worked on in LDS when both fit there (n <= lds_n), else in place.
__device__ void jacobi_orthogonalise(double* __restrict__ X, double* __restrict__ V, int32_t n, int* flag,
                                     double* lds, int32_t lds_n) {
    if (n <= lds_n) {
        double* Xl = lds;
        double* Vl = lds + (size_t)n * n;
        for (int32_t e = threadIdx.x; e < n * n; e += kCoreThreads) Xl[e] = X[e];
        jacobi_sweeps(Xl, Vl, n, flag);
        for (int32_t e = threadIdx.x; e < n * n; e += kCoreThreads) {
            X[e] = Xl[e];
            V[e] = Vl[e];
        }
        __syncthreads();
    } else {
        jacobi_sweeps(X, V, n, flag);
    }
}

__device__ void jacobi_sweeps(double* __restrict__ X, double* __restrict__ V, int32_t n, int* flag /*LDS*/) {
    const int tid = threadIdx.x;
    for (int32_t e = tid; e < n * n; e += kCoreThreads) V[e] = (e / n == e % n) ? 1.0 : 0.0;
    const int32_t h = (n + 1) / 2, m = 2 * h;          // m players; player n (if n is odd) sits out
    int T = 64;                                         // threads per pair: a power of two inside a wavefront
    while (T > 1 && h * T > kCoreThreads) T >>= 1;
    const int32_t pair = tid / T, sub = tid % T;
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        __syncthreads();
        if (tid == 0) *flag = 0;
        __syncthreads();
        for (int32_t round = 0; round < m - 1; ++round) {
            // circle method: player m-1 stays, the others move round; every two players meet once a sweep
            int32_t p = -1, q = -1;
            if (pair < h) {
                if (pair == 0) { p = m - 1; q = round; }
                else { p = (round + pair) % (m - 1); q = (round - pair + (m - 1)) % (m - 1); }
                if (p > q) { const int32_t t = p; p = q; q = t; }
            }
            const bool live = pair < h && q < n;
            double alpha = 0.0, beta = 0.0, gamma = 0.0;
            if (live) {
                const double* xp = X + (size_t)p * n;
                const double* xq = X + (size_t)q * n;
#pragma unroll 8
                for (int32_t row = sub; row < n; row += T) {
                    const double a = xp[row], b = xq[row];
                    alpha += a * a;
                    beta += b * b;
                    gamma += a * b;
                }
            }
            for (int off = T >> 1; off >= 1; off >>= 1) {     // the T lanes of a pair are neighbours
                alpha += __shfl_xor(alpha, off);
                beta += __shfl_xor(beta, off);
                gamma += __shfl_xor(gamma, off);
            }
            if (live && fabs(gamma) > kRotTol * sqrt(alpha * beta) && alpha * beta > 0.0) {
                const double zeta = (beta - alpha) / (2.0 * gamma);
                const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
                double* xp = X + (size_t)p * n;
                double* xq = X + (size_t)q * n;
                double* vp = V + (size_t)p * n;
                double* vq = V + (size_t)q * n;
#pragma unroll 8
                for (int32_t row = sub; row < n; row += T) {
                    const double a = xp[row], b = xq[row];
                    xp[row] = c * a - s * b;
                    xq[row] = s * a + c * b;
                    const double va = vp[row], vb = vq[row];
                    vp[row] = c * va - s * vb;
                    vq[row] = s * va + c * vb;
                }
                *flag = 1;
            }
            __syncthreads();
        }
        if (*flag == 0) break;           // read after the round's barrier; reset only after the next one
    }
    __syncthreads();
}

// norms of the columns of X into out[]
__device__ void column_norms(const double* __restrict__ X, int32_t n, double* __restrict__ out) {
    for (int32_t c = threadIdx.x; c < n; c += kCoreThreads) {
        double acc = 0.0;
        for (int32_t row = 0; row < n; ++row) acc += X[(size_t)c * n + row] * X[(size_t)c * n + row];
        out[c] = sqrt(acc);
    }
    __syncthreads();
}

__device__ double max_of(const double* v, int32_t n, double* red /*LDS[kCoreThreads/64]*/) {
    double mx = 0.0;
    for (int32_t i = threadIdx.x; i < n; i += kCoreThreads) mx = fmax(mx, v[i]);
    for (int off = 32; off >= 1; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    double all = 0.0;
    for (int w = 0; w < kCoreThreads / 64; ++w) all = fmax(all, red[w]);
    return all;
}

__global__ void __launch_bounds__(kCoreThreads)
ladder_core_kernel(int32_t r, LadderWs ws, double* __restrict__ sigma_out, int32_t lds_n) {
    extern __shared__ double lds[];               // two lds_n x lds_n matrices
    __shared__ int flag;
    __shared__ double red[kCoreThreads / 64];
    const int tid = threadIdx.x;
    // the Gram matrices: slabs added in slab order
    for (int32_t e = tid; e < r * r; e += kCoreThreads) {
        double a = 0.0, b = 0.0;
        for (int32_t p = 0; p < ws.slabs; ++p) {
            a += ws.PA[(size_t)p * r * r + e];
            b += ws.PB[(size_t)p * r * r + e];
        }
        ws.GA[e] = a;
        ws.GB[e] = b;
    }
    __syncthreads();
    // eigen-decompositions of the two Gram matrices
    jacobi_orthogonalise(ws.GA, ws.VA, r, &flag, lds, lds_n);
    column_norms(ws.GA, r, ws.lamA);
    jacobi_orthogonalise(ws.GB, ws.VB, r, &flag, lds, lds_n);
    column_norms(ws.GB, r, ws.lamB);
    const double lamA_max = max_of(ws.lamA, r, red), lamB_max = max_of(ws.lamB, r, red);
    // core M = L_A^1/2 V_A^T V_B L_B^1/2 (column-major), zero in the directions that carry nothing
    for (int32_t e = tid; e < r * r; e += kCoreThreads) {
        const int32_t i = e % r, j = e / r;
        const double la = ws.lamA[i], lb = ws.lamB[j];
        double v = 0.0;
        if (la > kEigTol * lamA_max && lb > kEigTol * lamB_max) {
            double acc = 0.0;
            for (int32_t k = 0; k < r; ++k) acc += ws.VA[(size_t)i * r + k] * ws.VB[(size_t)j * r + k];
            v = sqrt(la) * acc * sqrt(lb);
        }
        ws.M[e] = v;
    }
    __syncthreads();
    jacobi_orthogonalise(ws.M, ws.VM, r, &flag, lds, lds_n);      // M <- Y = U S
    column_norms(ws.M, r, ws.sig);
    const double sig_max = max_of(ws.sig, r, red);
    // rank of every column by descending singular value (ties by column index)
    // (a NaN norm, from NaN in the inputs, is ranked as +inf, so that the ranks are a permutation whatever the data)
    for (int32_t c = tid; c < r; c += kCoreThreads) {
        const double raw = ws.sig[c];
        const double mine = raw == raw ? raw : INFINITY;
        int32_t rank = 0;
        for (int32_t u = 0; u < r; ++u) {
            const double w = ws.sig[u];
            const double v = w == w ? w : INFINITY;
            rank += (v > mine || (v == mine && u < c)) ? 1 : 0;
        }
        ws.perm[rank] = c;
    }
    __syncthreads();
    for (int32_t i = tid; i < r; i += kCoreThreads) {
        const double s = ws.sig[ws.perm[i]];
        sigma_out[i] = s > kSigTol * sig_max ? s : 0.0;
    }
    // Z_A[j][i] = L_A^-1/2[j] Y[j][perm i] S^-1/2[perm i]  (into GA's storage, column-major),
    // Z_B[j][i] = L_B^-1/2[j] V[j][perm i] S^+1/2[perm i]  (into GB's storage)
    for (int32_t e = tid; e < r * r; e += kCoreThreads) {
        const int32_t j = e % r, i = e / r, c = ws.perm[i];
        const double s = ws.sig[c];
        const bool keep = s > kSigTol * sig_max && s > 0.0;
        const double la = ws.lamA[j], lb = ws.lamB[j];
        const double ia = la > kEigTol * lamA_max ? 1.0 / sqrt(la) : 0.0;
        const double ib = lb > kEigTol * lamB_max ? 1.0 / sqrt(lb) : 0.0;
        ws.GA[e] = keep ? ia * ws.M[(size_t)c * r + j] / sqrt(s) : 0.0;
        ws.GB[e] = keep ? ib * ws.VM[(size_t)c * r + j] * sqrt(s) : 0.0;
    }
    __syncthreads();
    // T_A[k][i] = sum_j V_A[k][j] Z_A[j][i],  T_B[k][i] = sum_j V_B[k][j] Z_B[j][i]
    for (int32_t e = tid; e < r * r; e += kCoreThreads) {
        const int32_t i = e % r, k = e / r;
        double ta = 0.0, tb = 0.0;
        for (int32_t j = 0; j < r; ++j) {
            ta += ws.VA[(size_t)j * r + k] * ws.GA[(size_t)i * r + j];
            tb += ws.VB[(size_t)j * r + k] * ws.GB[(size_t)i * r + j];
        }
        ws.TA[(size_t)k * r + i] = ta;
        ws.TB[(size_t)k * r + i] = tb;
    }
}

// ---- 3. out(s, i) = sum_k in(s, k) T[k][i] over samples s; strides as in gram_kernel ----
constexpr int kApplySamples = 32;

__global__ void __launch_bounds__(256)
apply_map_kernel(const void* __restrict__ in, int bf16, int64_t n_samples, int64_t ss, int64_t cs, int32_t r,
                 const double* __restrict__ T, void* __restrict__ out, int64_t oss, int64_t ocs) {
    extern __shared__ float tile[];                      // [kApplySamples][r + 1], input then output
    const int tid = threadIdx.x;
    const int ld = r + 1;
    const int64_t s0 = (int64_t)blockIdx.x * kApplySamples;
    const bool comp_fast = cs == 1;
    for (int e = tid; e < kApplySamples * r; e += 256) {
        const int c = comp_fast ? (e % r) : (e / kApplySamples);
        const int s = comp_fast ? (e / r) : (e % kApplySamples);
        tile[s * ld + c] = (s0 + s < n_samples) ? load_elem(in, (s0 + s) * ss + (int64_t)c * cs, bf16) : 0.0f;
    }
    __syncthreads();
    double acc[kApplySamples];
#pragma unroll
    for (int s = 0; s < kApplySamples; ++s) acc[s] = 0.0;
    if (tid < r) {
        for (int32_t k = 0; k < r; ++k) {
            const double t = T[(size_t)k * r + tid];
#pragma unroll
            for (int s = 0; s < kApplySamples; ++s) acc[s] += (double)tile[s * ld + k] * t;
        }
    }
    __syncthreads();
    if (tid < r) {
#pragma unroll
        for (int s = 0; s < kApplySamples; ++s) tile[s * ld + tid] = (float)acc[s];
    }
    __syncthreads();
    const bool out_comp_fast = ocs == 1;
    for (int e = tid; e < kApplySamples * r; e += 256) {
        const int c = out_comp_fast ? (e % r) : (e / kApplySamples);
        const int s = out_comp_fast ? (e / r) : (e % kApplySamples);
        if (s0 + s < n_samples) store_elem(out, (s0 + s) * oss + (int64_t)c * ocs, tile[s * ld + c], bf16);
    }
}

}  // namespace
}  // namespace cwl

using namespace cwl;

extern "C" size_t cwl_ladder_workspace_bytes(int32_t r) {
    if (r < 1 || r > CWL_MAX_RANK) return 0;
    return ladder_ws_layout(r, nullptr, nullptr);
}

extern "C" cwl_status cwl_build_ladder(cwl_dtype dt, const void* A, int64_t lda, const void* B, int64_t ldb,
                                       int64_t d_in, int64_t d_out, int32_t r, void* A_out, int64_t lda_out,
                                       void* B_out, int64_t ldb_out, double* sigma, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    if (dt != CWL_F32 && dt != CWL_BF16) return CWL_ERR_INVALID_ARG;
    if (r < 1 || r > CWL_MAX_RANK || d_in < 1 || d_out < 1) return CWL_ERR_INVALID_ARG;
    if (d_in >= (int64_t)1 << 31 || d_out >= (int64_t)1 << 31) return CWL_ERR_INVALID_ARG;
    if (lda < r || lda_out < r || ldb < d_out || ldb_out < d_out) return CWL_ERR_INVALID_ARG;
    if (!A || !B || !A_out || !B_out || !sigma || !workspace) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return CWL_ERR_INVALID_ARG;
    LadderWs ws;
    if (workspace_bytes < ladder_ws_layout(r, workspace, &ws)) return CWL_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int bf16 = dt == CWL_BF16 ? 1 : 0;
    const unsigned tiles = (unsigned)((r + kGramTile - 1) / kGramTile);
    gram_kernel<<<dim3(tiles, tiles, (unsigned)ws.slabs), dim3(256), 0, s>>>(A, bf16, d_in, lda, 1, r, ws.PA);
    CWL_RETURN_IF_LAUNCH_FAILED();
    gram_kernel<<<dim3(tiles, tiles, (unsigned)ws.slabs), dim3(256), 0, s>>>(B, bf16, d_out, 1, ldb, r, ws.PB);
    CWL_RETURN_IF_LAUNCH_FAILED();
    // the r x r matrices of a decomposition are worked on in LDS when two of them fit into 144 KiB (r <= 96)
    constexpr size_t kCoreLdsMax = 144 * 1024;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(ladder_core_kernel), (int)kCoreLdsMax, lds_set) != CWL_OK)
        return CWL_ERR_DEVICE;
    const size_t core_lds = 2 * sizeof(double) * (size_t)r * (size_t)r;
    const bool in_lds = core_lds <= kCoreLdsMax;
    ladder_core_kernel<<<dim3(1), dim3(kCoreThreads), in_lds ? core_lds : 0, s>>>(r, ws, sigma, in_lds ? r : 0);
    CWL_RETURN_IF_LAUNCH_FAILED();
    const size_t lds = sizeof(float) * (size_t)kApplySamples * (size_t)(r + 1);
    apply_map_kernel<<<dim3((unsigned)((d_in + kApplySamples - 1) / kApplySamples)), dim3(256), lds, s>>>(
        A, bf16, d_in, lda, 1, r, ws.TA, A_out, lda_out, 1);
    CWL_RETURN_IF_LAUNCH_FAILED();
    apply_map_kernel<<<dim3((unsigned)((d_out + kApplySamples - 1) / kApplySamples)), dim3(256), lds, s>>>(
        B, bf16, d_out, 1, ldb, r, ws.TB, B_out, 1, ldb_out);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
