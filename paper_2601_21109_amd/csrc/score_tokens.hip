// cwl_score_tokens: row-wise softmax entropy of the logits (Sec. III-A signal (i), Sec. IV-A of
// arxiv 2601.21109).  One pass over the logits; HBM-bandwidth bound.
//
// Each thread streams 16-byte vectors of its row and keeps an online state (c, S, W) in the
// log2 domain:  S = sum 2^(z*L - c),  W = sum (z*L - c) 2^(z*L - c),  L = log2(e), c = the
// offset in use (about max(z)*L).  When a larger logit arrives the state is rescaled.  States
// are merged across the lanes of a wavefront with shuffles and across wavefronts through LDS,
// always in the same order, so results are reproducible.  H = ln2 * (log2 S - W / S).
// fp32 throughout: the absolute error of H is a few 2^-24 * (1 + |log2 S| + |W / S|), so very
// peaked rows (H below about 0.05 nat) are resolved to ~1e-7 nat absolute, not 1e-5 relative.
#include "common.h"

namespace {

constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

struct EntState {
    float c, S, W;
};

__device__ __forceinline__ void ent_raise_offset(EntState& s, float c_new) {
    if (c_new > s.c) {
        // an empty state has c = -inf and S = W = 0: any finite factor keeps it empty
        const float d = (s.c == -INFINITY) ? 0.0f : s.c - c_new;
        const float f = __builtin_amdgcn_exp2f(d);
        s.W = f * (s.W + d * s.S);
        s.S = f * s.S;
        s.c = c_new;
    }
}

// Adds one logit to a state whose offset is `off` (= s.c, or 0 while the state is still empty so
// that a leading run of -inf logits does not form inf - inf).
__device__ __forceinline__ void ent_add(EntState& s, float off, float z) {
    const float t = fmaf(z, kLog2e, -off);
    const float e = __builtin_amdgcn_exp2f(t);
    s.S += e;                       // NaN, and +inf - +inf, poison S and with it the row
    // t = -inf has e = 0 and must add nothing: clamp t for the product only (2^-200 is 0 in fp32,
    // so no finite term changes)
    s.W = fmaf(fmaxf(t, -200.0f), e, s.W);
}

__device__ __forceinline__ void ent_merge(EntState& a, const EntState& b) {
    EntState bb = b;
    const float c = fmaxf(a.c, bb.c);
    ent_raise_offset(a, c);
    ent_raise_offset(bb, c);
    a.S += bb.S;
    a.W += bb.W;
}

template <typename T>
struct Vec;
template <>
struct Vec<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(const float* p, float (&z)[4]) {
        // streamed once: non-temporal, so the logits do not displace reusable lines from the caches
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        z[0] = v[0]; z[1] = v[1]; z[2] = v[2]; z[3] = v[3];
    }
    __device__ static __forceinline__ float one(const float* p) { return *p; }
};
template <>
struct Vec<uint16_t> {   // bf16 bit patterns
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const uint16_t* p, float (&z)[8]) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        const uint32_t w[4] = {v[0], v[1], v[2], v[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            z[2 * i] = __uint_as_float(w[i] << 16);
            z[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ float one(const uint16_t* p) {
        return __uint_as_float(((uint32_t)*p) << 16);
    }
};

template <int N>
__device__ __forceinline__ void ent_add_vec(EntState& s, float& m, const float (&z)[N]) {
    float vm = z[0];   // nested in threes so that the compiler forms v_max3_f32
#pragma unroll
    for (int i = 1; i + 1 < N; i += 2) vm = fmaxf(fmaxf(vm, z[i]), z[i + 1]);
    if (N % 2 == 0) vm = fmaxf(vm, z[N - 1]);
    if (vm > m) {
        m = vm;
        ent_raise_offset(s, vm * kLog2e);
    }
    const float off = (s.c == -INFINITY) ? 0.0f : s.c;
#pragma unroll
    for (int i = 0; i < N; ++i) ent_add(s, off, z[i]);
}

// WAVES wavefronts cooperate on one row.  WAVES = 1: a block of 256 threads holds 4 rows;
// otherwise one row per block of WAVES * 64 threads.
template <typename T, int WAVES>
__global__ void __launch_bounds__(WAVES >= 2 ? WAVES * 64 : 256)
score_tokens_kernel(const T* __restrict__ logits, int64_t n_rows, int64_t vocab,
                    int64_t row_stride, float* __restrict__ entropy) {
    constexpr int VEC = Vec<T>::N;
    constexpr int UNROLL = 4;
    constexpr int GROUP = WAVES * 64;                     // threads per row
    constexpr int ROWS_PER_BLOCK = (WAVES >= 2) ? 1 : 4;
    const int tid = threadIdx.x;
    const int g_tid = tid % GROUP;
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + tid / GROUP;
    const bool row_ok = row < n_rows;

    // two independent online states per thread: shorter dependency chains through S and W
    EntState s = {-INFINITY, 0.0f, 0.0f}, s2 = {-INFINITY, 0.0f, 0.0f};
    float m = -INFINITY, m2 = -INFINITY;
    if (row_ok) {
        const T* rp = logits + row * row_stride;
        // split the row into unaligned head, 16-byte vectors, tail
        const uintptr_t mis = (reinterpret_cast<uintptr_t>(rp) & 15u) / sizeof(T);
        int64_t head = mis ? (int64_t)(VEC - mis) : 0;
        if (head > vocab) head = vocab;
        const int64_t nvec = (vocab - head) / VEC;
        const int64_t tail0 = head + nvec * VEC;
        const T* vp = rp + head;

        int64_t i = g_tid;
        for (; i + (int64_t)(UNROLL - 1) * GROUP < nvec; i += (int64_t)UNROLL * GROUP) {
            float z[UNROLL][VEC];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) Vec<T>::load(vp + (i + (int64_t)u * GROUP) * VEC, z[u]);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                if (u & 1) ent_add_vec<VEC>(s2, m2, z[u]);
                else ent_add_vec<VEC>(s, m, z[u]);
            }
        }
        for (; i < nvec; i += GROUP) {
            float z[VEC];
            Vec<T>::load(vp + i * VEC, z);
            ent_add_vec<VEC>(s, m, z);
        }
        // head and tail elements, one per thread (at most 2*(VEC-1) of them)
        const int64_t n_loose = head + (vocab - tail0);
        if (g_tid < n_loose) {
            const int64_t idx = (g_tid < head) ? g_tid : tail0 + (g_tid - head);
            float z[1] = {Vec<T>::one(rp + idx)};
            ent_add_vec<1>(s, m, z);
        }
    }

    ent_merge(s, s2);
    // merge across the 64 lanes
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        EntState o;
        o.c = __shfl_xor(s.c, off);
        o.S = __shfl_xor(s.S, off);
        o.W = __shfl_xor(s.W, off);
        ent_merge(s, o);
    }
    if constexpr (WAVES > 1) {
        __shared__ EntState part[WAVES];
        const int wave = tid / 64;
        if ((tid & 63) == 0) part[wave] = s;
        __syncthreads();
        if (tid == 0) {
            s = part[0];
            for (int w = 1; w < WAVES; ++w) ent_merge(s, part[w]);
        }
    }
    if (row_ok && g_tid == 0) {
        entropy[row] = kLn2 * (log2f(s.S) - s.W / s.S);
    }
}

template <typename T>
cwl_status launch(const void* logits, int64_t n_rows, int64_t vocab, int64_t row_stride,
                  float* entropy, hipStream_t st) {
    const int64_t row_bytes = vocab * (int64_t)sizeof(T);
    const T* lp = static_cast<const T*>(logits);
    cwl::prof_begin(CWL_PROF_SCORE, st);
    // threads per row: enough 16-byte loads per thread to amortise the state merge, enough
    // blocks per CU to keep HBM busy (measured best on 64 KB rows: 2 wavefronts per row)
    if (n_rows <= 128 && row_bytes > 16 * 1024) {
        // a decode step's handful of rows: one workgroup per row is all the parallelism there is,
        // so give every row sixteen wavefronts
        score_tokens_kernel<T, 16><<<dim3((unsigned)n_rows), dim3(1024), 0, st>>>(lp, n_rows, vocab, row_stride, entropy);
    } else if (row_bytes <= 16 * 1024) {
        const int64_t blocks = (n_rows + 3) / 4;
        score_tokens_kernel<T, 1><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(lp, n_rows, vocab, row_stride, entropy);
    } else if (row_bytes <= 128 * 1024) {
        score_tokens_kernel<T, 2><<<dim3((unsigned)n_rows), dim3(128), 0, st>>>(lp, n_rows, vocab, row_stride, entropy);
    } else if (row_bytes <= 512 * 1024) {
        score_tokens_kernel<T, 4><<<dim3((unsigned)n_rows), dim3(256), 0, st>>>(lp, n_rows, vocab, row_stride, entropy);
    } else {
        score_tokens_kernel<T, 16><<<dim3((unsigned)n_rows), dim3(1024), 0, st>>>(lp, n_rows, vocab, row_stride, entropy);
    }
    cwl::prof_end(CWL_PROF_SCORE, st);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace

extern "C" cwl_status cwl_score_tokens(const void* logits, cwl_dtype dt, int64_t n_rows,
                                       int64_t vocab, int64_t row_stride, float* entropy,
                                       void* stream) {
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || vocab < 1 || row_stride < vocab)
        return CWL_ERR_INVALID_ARG;
    if (dt != CWL_F32 && dt != CWL_BF16) return CWL_ERR_INVALID_ARG;
    if (n_rows == 0) return CWL_OK;
    if (!logits || !entropy) return CWL_ERR_NULL;
    const size_t esize = dt == CWL_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(logits) % esize) return CWL_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == CWL_F32) return launch<float>(logits, n_rows, vocab, row_stride, entropy, st);
    return launch<uint16_t>(logits, n_rows, vocab, row_stride, entropy, st);
}
