// cwl_kv_quantise_chunks / cwl_kv_dequantise: the chunk-level KV-cache policy (Sec. III-E, the
// KV-cache policy controller, and Sec. IV-F of arxiv 2601.21109): rows of easy chunks are stored in
// INT8 with one fp32 scale per row and head, rows of the other chunks at full fidelity, in two pools.
// Streaming work, bound by reading the cache rows once from HBM.
//
//   kv_plan_slot_kernel  tables of up to 4096 chunks: the two kernels below in one launch (every workgroup
//                        scans the chunk list itself and keeps it in LDS)
//   kv_plan_kernel       one workgroup: per chunk its policy and its first row in its pool (two
//                        exclusive scans over the chunk lengths, in table order), the pool totals
//   kv_slot_kernel       one thread per row: the row's chunk (binary search in the ascending chunk
//                        starts) and with it its slot.  A kernel of its own because the search is a
//                        chain of dependent look-ups: in front of every wavefront's stores it made the
//                        streaming kernel wait 8 round trips per row (120 us for 16384 rows of 8 KB);
//                        here all rows wait at once
//   kv_quantise_kernel   one wavefront per row: 16-byte loads, the maximum of a head over the lanes
//                        that hold it, codes packed eight to a lane
//   kv_dequantise_kernel one wavefront per row: the row read back as bf16
#include "common.h"

namespace {

using cwl::kWave;

constexpr int kPlanThreads = 1024;
constexpr int kRowsPerBlock = 4;        // wavefronts per workgroup (one per row, or per row segment)
constexpr int kMaxPasses = 16;          // 512 elements per pass: rows of up to 8192 elements

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

struct KvShape {
    int32_t n_heads, head_dim, k_keep;
    int32_t width;           // n_heads * head_dim
    int32_t lanes_per_head;  // head_dim / 8: a power of two, 4 .. 64
};

// ---- plan ---------------------------------------------------------------------------------------
// chunk_slot[c] >= 0: first row of chunk c in the INT8 pool; <= -1: first row -1 - chunk_slot[c] in the
// full pool.  Pool rows are handed out in table order, so the scans run over the chunks as they are listed.
__global__ void __launch_bounds__(kPlanThreads)
kv_plan_kernel(const int32_t* __restrict__ chunk_offsets, int32_t n_seqs, const int32_t* __restrict__ chunk_len,
               const int32_t* __restrict__ rank_idx, int32_t chunk_cap, int32_t k_keep,
               int64_t cap_q, int64_t cap_f, int32_t* __restrict__ chunk_slot, int32_t* __restrict__ n_chunks_out,
               int32_t* __restrict__ counts, int32_t* __restrict__ status_word) {
    __shared__ int64_t wave_q[kPlanThreads / 64], wave_f[kPlanThreads / 64];
    __shared__ int64_t carry_q_sh, carry_f_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t n_chunks = chunk_offsets[n_seqs];
    if (n_chunks > chunk_cap) n_chunks = chunk_cap;
    if (n_chunks < 0) n_chunks = 0;
    if (tid == 0) {
        carry_q_sh = 0;
        carry_f_sh = 0;
        *n_chunks_out = n_chunks;
    }
    __syncthreads();
    for (int32_t c0 = 0; c0 < n_chunks; c0 += kPlanThreads) {
        const int32_t c = c0 + tid;
        int64_t lq = 0, lf = 0;
        bool easy = false;
        if (c < n_chunks) {
            const int32_t k = rank_idx[c];
            int32_t len = chunk_len[c];
            if (len < 0) len = 0;
            easy = k >= 0 && k < k_keep;
            (easy ? lq : lf) = len;
        }
        int64_t iq = lq, ifl = lf;                 // inclusive scans inside the wavefront
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t vq = cwl::shfl_up_i64(iq, off), vf = cwl::shfl_up_i64(ifl, off);
            if (lane >= off) {
                iq += vq;
                ifl += vf;
            }
        }
        if (lane == 63) {
            wave_q[wave] = iq;
            wave_f[wave] = ifl;
        }
        __syncthreads();
        int64_t base_q = carry_q_sh, base_f = carry_f_sh, tot_q = 0, tot_f = 0;
        for (int w = 0; w < kPlanThreads / 64; ++w) {
            if (w < wave) {
                base_q += wave_q[w];
                base_f += wave_f[w];
            }
            tot_q += wave_q[w];
            tot_f += wave_f[w];
        }
        if (c < n_chunks) {
            const int64_t first = easy ? base_q + iq - lq : base_f + ifl - lf;
            // rows beyond 2^31 cannot be addressed by a slot; such a table is rejected on the host (n_rows < 2^31)
            chunk_slot[c] = easy ? (int32_t)first : (int32_t)(-1 - first);
        }
        __syncthreads();
        if (tid == 0) {
            carry_q_sh += tot_q;
            carry_f_sh += tot_f;
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int64_t q = carry_q_sh, f = carry_f_sh;
        counts[0] = q > 0x7fffffffll ? 0x7fffffff : (int32_t)q;
        counts[1] = f > 0x7fffffffll ? 0x7fffffff : (int32_t)f;
        // a pool is too small exactly when its chunks list more rows than it holds
        *status_word = (q > cap_q || f > cap_f) ? (int32_t)CWL_STATUS_CAPACITY : 0;
    }
}

// ---- quantise -----------------------------------------------------------------------------------
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ int32_t code_of(float x, float inv) {
    const float v = x * inv;
    if (!(v == v)) return 0;                          // a NaN element (or inf * 0) has code 0
    const float r = rintf(v);                         // nearest, ties to even
    return r > 127.0f ? 127 : (r < -127.0f ? -127 : (int32_t)r);
}

__global__ void __launch_bounds__(256)
kv_slot_kernel(int64_t n_rows, const int32_t* __restrict__ chunk_start, const int32_t* __restrict__ chunk_len,
               const int32_t* __restrict__ chunk_slot, const int32_t* __restrict__ n_chunks_p, int64_t cap_q,
               int64_t cap_f, int32_t* __restrict__ slot) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_rows) return;
    // chunk of the row: the last chunk whose start is <= t (starts ascend in the chunker's table)
    const int32_t n_chunks = *n_chunks_p;
    int32_t lo = 0, hi = n_chunks;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if ((int64_t)chunk_start[mid] <= t) lo = mid + 1; else hi = mid;
    }
    const int32_t c = lo - 1;
    int32_t my_slot = INT32_MIN;
    if (c >= 0) {
        const int64_t j = t - chunk_start[c];
        if (j < chunk_len[c]) {
            const int32_t cs = chunk_slot[c];
            const int64_t idx = (cs >= 0 ? (int64_t)cs : -1 - (int64_t)cs) + j;
            if (cs >= 0) {
                if (idx < cap_q) my_slot = (int32_t)idx;
            } else if (idx < cap_f) {
                my_slot = (int32_t)(-1 - idx);
            }
        }
    }
    slot[t] = my_slot;
}

// Plan and slots in one launch, for tables of up to kFusedChunks chunks: every workgroup of 256 rows scans the
// whole chunk list itself (a few hundred entries; starts, lengths and first pool rows stay in LDS) and then
// searches its rows' chunks there, so a row waits for two round trips to memory instead of a launch boundary
// and eight.  Workgroup 0 also writes the pool totals and the status word.
constexpr int kFusedChunks = 4096;

__global__ void __launch_bounds__(256)
kv_plan_slot_kernel(int64_t n_rows, const int32_t* __restrict__ chunk_offsets, int32_t n_seqs,
                    const int32_t* __restrict__ chunk_start, const int32_t* __restrict__ chunk_len,
                    const int32_t* __restrict__ rank_idx, int32_t chunk_cap, int32_t k_keep, int64_t cap_q,
                    int64_t cap_f, int32_t* __restrict__ slot, int32_t* __restrict__ counts,
                    int32_t* __restrict__ status_word) {
    __shared__ int32_t s_start[kFusedChunks], s_len[kFusedChunks], s_slot[kFusedChunks];
    __shared__ int64_t wave_q[4], wave_f[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t n_chunks = chunk_offsets[n_seqs];
    if (n_chunks > chunk_cap) n_chunks = chunk_cap;
    if (n_chunks < 0) n_chunks = 0;
    int64_t carry_q = 0, carry_f = 0;              // the same in every thread
    for (int32_t c0 = 0; c0 < n_chunks; c0 += 256) {
        const int32_t c = c0 + tid;
        int64_t lq = 0, lf = 0;
        bool easy = false;
        if (c < n_chunks) {
            const int32_t k = rank_idx[c];
            const int32_t len_raw = chunk_len[c];
            s_start[c] = chunk_start[c];
            s_len[c] = len_raw;
            easy = k >= 0 && k < k_keep;
            (easy ? lq : lf) = len_raw < 0 ? 0 : len_raw;
        }
        int64_t iq = lq, ifl = lf;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t vq = cwl::shfl_up_i64(iq, off), vf = cwl::shfl_up_i64(ifl, off);
            if (lane >= off) {
                iq += vq;
                ifl += vf;
            }
        }
        if (lane == 63) {
            wave_q[wave] = iq;
            wave_f[wave] = ifl;
        }
        __syncthreads();
        int64_t base_q = carry_q, base_f = carry_f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) {
                base_q += wave_q[w];
                base_f += wave_f[w];
            }
            carry_q += wave_q[w];
            carry_f += wave_f[w];
        }
        if (c < n_chunks) {
            const int64_t first = easy ? base_q + iq - lq : base_f + ifl - lf;
            s_slot[c] = easy ? (int32_t)first : (int32_t)(-1 - first);
        }
        __syncthreads();                           // the wavefront totals are rewritten by the next round
    }
    if (blockIdx.x == 0 && tid == 0) {
        counts[0] = carry_q > 0x7fffffffll ? 0x7fffffff : (int32_t)carry_q;
        counts[1] = carry_f > 0x7fffffffll ? 0x7fffffff : (int32_t)carry_f;
        *status_word = (carry_q > cap_q || carry_f > cap_f) ? (int32_t)CWL_STATUS_CAPACITY : 0;
    }
    const int64_t t = (int64_t)blockIdx.x * 256 + tid;
    if (t >= n_rows) return;
    int32_t lo = 0, hi = n_chunks;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if ((int64_t)s_start[mid] <= t) lo = mid + 1; else hi = mid;
    }
    const int32_t c = lo - 1;
    int32_t my_slot = INT32_MIN;
    if (c >= 0) {
        const int64_t j = t - s_start[c];
        if (j < s_len[c]) {
            const int32_t cs = s_slot[c];
            const int64_t idx = (cs >= 0 ? (int64_t)cs : -1 - (int64_t)cs) + j;
            if (cs >= 0) {
                if (idx < cap_q) my_slot = (int32_t)idx;
            } else if (idx < cap_f) {
                my_slot = (int32_t)(-1 - idx);
            }
        }
    }
    slot[t] = my_slot;
}

// A wavefront takes a segment of PASSES * 512 elements of one row (whole heads: a head has at most 512
// elements), `segs` segments per row.  PASSES is a compile-time constant of at most four: the segment lives
// in registers between its loads and its stores; with a run-time bound on these loops it went through
// scratch memory, and eight passes at once took 231 registers (two wavefronts per SIMD).
template <int PASSES>
__global__ void __launch_bounds__(kRowsPerBlock * 64)
kv_quantise_kernel(const uint16_t* __restrict__ kv, int64_t ld, int64_t n_rows, KvShape sh, int32_t segs,
                   const int32_t* __restrict__ slot, int8_t* __restrict__ q_codes, float* __restrict__ q_scale,
                   uint16_t* __restrict__ f_pool) {
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int64_t t = w / segs;
    if (t >= n_rows) return;
    const int seg0 = (int)(w % segs) * PASSES * 512;
    const int32_t my_slot = slot[t];
    u32x4 v[PASSES];
    const uint16_t* rp = kv + t * ld;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int e0 = seg0 + p * 512 + lane * 8;
        v[p] = u32x4{0u, 0u, 0u, 0u};
        if (e0 < sh.width) v[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(rp + e0));
    }
    if (my_slot == INT32_MIN) return;
    if (my_slot < 0) {
        uint16_t* dst = f_pool + (int64_t)(-1 - my_slot) * sh.width;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int e0 = seg0 + p * 512 + lane * 8;
            if (e0 < sh.width) *reinterpret_cast<u32x4*>(dst + e0) = v[p];
        }
        return;
    }
    int8_t* crow = q_codes + (int64_t)my_slot * sh.width;
    float* srow = q_scale + (int64_t)my_slot * sh.n_heads;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int e0 = seg0 + p * 512 + lane * 8;
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = lo_bf16(v[p][i]);
            x[2 * i + 1] = hi_bf16(v[p][i]);
        }
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(x[i]));      // fmaxf drops a NaN operand
        for (int off = 1; off < sh.lanes_per_head; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        const float inv = amax > 0.0f ? __fdiv_rn(127.0f, amax) : 0.0f;
        if (e0 < sh.width) {
            uint32_t w0 = 0, w1 = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                w0 |= ((uint32_t)code_of(x[i], inv) & 0xffu) << (8 * i);
                w1 |= ((uint32_t)code_of(x[4 + i], inv) & 0xffu) << (8 * i);
            }
            *reinterpret_cast<u32x2*>(crow + e0) = u32x2{w0, w1};
            if ((lane & (sh.lanes_per_head - 1)) == 0) srow[e0 / sh.head_dim] = __fdiv_rn(amax, 127.0f);
        }
    }
}

// ---- dequantise ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(kRowsPerBlock * 64)
kv_dequantise_kernel(const int32_t* __restrict__ slot, int64_t n_rows, const int8_t* __restrict__ q_codes,
                     const float* __restrict__ q_scale, const uint16_t* __restrict__ f_pool, KvShape sh,
                     uint16_t* __restrict__ out, int64_t ld_out) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (t >= n_rows) return;
    const int32_t s = slot[t];
    uint16_t* dst = out + t * ld_out;
    const int passes = (sh.width + 511) / 512;
    for (int p = 0; p < passes; ++p) {
        const int e0 = p * 512 + lane * 8;
        if (e0 >= sh.width) break;
        u32x4 o = {0u, 0u, 0u, 0u};
        if (s == INT32_MIN) {
            // not cached: zeros
        } else if (s < 0) {
            o = *reinterpret_cast<const u32x4*>(f_pool + (int64_t)(-1 - s) * sh.width + e0);
        } else {
            const u32x2 w = *reinterpret_cast<const u32x2*>(q_codes + (int64_t)s * sh.width + e0);
            const float sc = q_scale[(int64_t)s * sh.n_heads + e0 / sh.head_dim];
            float y[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                y[i] = (float)(int8_t)((w[0] >> (8 * i)) & 0xffu) * sc;
                y[4 + i] = (float)(int8_t)((w[1] >> (8 * i)) & 0xffu) * sc;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const __bf16 a = (__bf16)y[2 * i], b = (__bf16)y[2 * i + 1];      // nearest, ties to even
                o[i] = (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
            }
        }
        *reinterpret_cast<u32x4*>(dst + e0) = o;
    }
}

cwl_status check_shape(const cwl_kv_params* p, KvShape* sh) {
    if (!p) return CWL_ERR_NULL;
    if (p->n_heads < 1 || p->head_dim < 1 || p->k_keep < 0) return CWL_ERR_INVALID_ARG;
    const int64_t width = (int64_t)p->n_heads * p->head_dim;
    const int l = p->head_dim / 8;
    if (p->head_dim % 8 != 0 || l < 4 || l > 64 || (l & (l - 1)) != 0 || width > 512 * kMaxPasses)
        return CWL_ERR_UNSUPPORTED;
    sh->n_heads = p->n_heads;
    sh->head_dim = p->head_dim;
    sh->k_keep = p->k_keep;
    sh->width = (int32_t)width;
    sh->lanes_per_head = l;
    return CWL_OK;
}

}  // namespace

extern "C" size_t cwl_kv_workspace_bytes(int32_t chunk_cap) {
    if (chunk_cap < 0) return 0;
    return cwl::align_up(sizeof(int32_t) * ((size_t)chunk_cap + 1), 256) + 256;
}

extern "C" cwl_status cwl_kv_quantise_chunks(const void* kv, int64_t ld, int64_t n_rows, const int32_t* chunk_offsets,
                                             int32_t n_seqs, const int32_t* chunk_start, const int32_t* chunk_len,
                                             const int32_t* rank_idx, int32_t chunk_cap, const cwl_kv_params* p,
                                             int32_t* slot, int32_t* counts, int8_t* q_codes, float* q_scale,
                                             int64_t cap_q, void* f_pool, int64_t cap_f, int32_t* status_word,
                                             void* workspace, size_t workspace_bytes, void* stream) {
    KvShape sh;
    const cwl_status cs = check_shape(p, &sh);
    if (cs != CWL_OK) return cs;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0 || chunk_cap < 0 || cap_q < 0 || cap_f < 0 ||
        ld < sh.width)
        return CWL_ERR_INVALID_ARG;
    if (!chunk_offsets || !counts || !status_word || !workspace) return CWL_ERR_NULL;
    if (chunk_cap > 0 && (!chunk_start || !chunk_len || !rank_idx)) return CWL_ERR_NULL;
    if (n_rows > 0 && (!kv || !slot)) return CWL_ERR_NULL;
    if (cap_q > 0 && (!q_codes || !q_scale)) return CWL_ERR_NULL;
    if (cap_f > 0 && !f_pool) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return CWL_ERR_INVALID_ARG;
    if (workspace_bytes < cwl_kv_workspace_bytes(chunk_cap)) return CWL_ERR_CAPACITY;
    if (ld % 8 != 0 || reinterpret_cast<uintptr_t>(kv) % 16 || reinterpret_cast<uintptr_t>(f_pool) % 16 ||
        reinterpret_cast<uintptr_t>(q_codes) % 8)
        return CWL_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t* chunk_slot = static_cast<int32_t*>(workspace);
    int32_t* n_chunks_dev = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) +
                                                       cwl::align_up(sizeof(int32_t) * ((size_t)chunk_cap + 1), 256));
    cwl::prof_begin(CWL_PROF_KV, st);
    const unsigned row_blocks = (unsigned)((n_rows + 255) / 256);
    if (chunk_cap <= kFusedChunks) {
        kv_plan_slot_kernel<<<dim3(row_blocks > 0 ? row_blocks : 1), dim3(256), 0, st>>>(
            n_rows, chunk_offsets, n_seqs, chunk_start, chunk_len, rank_idx, chunk_cap, sh.k_keep, cap_q, cap_f, slot,
            counts, status_word);
    } else {
        kv_plan_kernel<<<dim3(1), dim3(kPlanThreads), 0, st>>>(chunk_offsets, n_seqs, chunk_len, rank_idx, chunk_cap,
                                                                sh.k_keep, cap_q, cap_f, chunk_slot, n_chunks_dev,
                                                                counts, status_word);
        CWL_RETURN_IF_LAUNCH_FAILED();
        if (n_rows > 0)
            kv_slot_kernel<<<dim3(row_blocks), dim3(256), 0, st>>>(n_rows, chunk_start, chunk_len, chunk_slot,
                                                                   n_chunks_dev, cap_q, cap_f, slot);
    }
    CWL_RETURN_IF_LAUNCH_FAILED();
    if (n_rows > 0) {
        const int passes = (sh.width + 511) / 512;
        const int per_wave = passes >= 4 ? 4 : (passes >= 2 ? 2 : 1);
        const int32_t segs = (passes + per_wave - 1) / per_wave;
        const int64_t waves = n_rows * segs;
        const unsigned blocks = (unsigned)((waves + kRowsPerBlock - 1) / kRowsPerBlock);
#define CWL_KV_LAUNCH(P)                                                                                  \
    kv_quantise_kernel<P><<<dim3(blocks), dim3(kRowsPerBlock * 64), 0, st>>>(                             \
        static_cast<const uint16_t*>(kv), ld, n_rows, sh, segs, slot, q_codes, q_scale, static_cast<uint16_t*>(f_pool))
        if (per_wave == 1) CWL_KV_LAUNCH(1);
        else if (per_wave == 2) CWL_KV_LAUNCH(2);
        else CWL_KV_LAUNCH(4);
#undef CWL_KV_LAUNCH
    }
    cwl::prof_end(CWL_PROF_KV, st);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

extern "C" cwl_status cwl_kv_dequantise(const int32_t* slot, int64_t n_rows, const int8_t* q_codes,
                                        const float* q_scale, const void* f_pool, const cwl_kv_params* p, void* out,
                                        int64_t ld_out, void* stream) {
    KvShape sh;
    const cwl_status cs = check_shape(p, &sh);
    if (cs != CWL_OK) return cs;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || ld_out < sh.width) return CWL_ERR_INVALID_ARG;
    if (n_rows == 0) return CWL_OK;
    if (!slot || !out) return CWL_ERR_NULL;
    if (ld_out % 8 != 0 || reinterpret_cast<uintptr_t>(out) % 16 || reinterpret_cast<uintptr_t>(f_pool) % 16 ||
        reinterpret_cast<uintptr_t>(q_codes) % 8)
        return CWL_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned blocks = (unsigned)((n_rows + kRowsPerBlock - 1) / kRowsPerBlock);
    kv_dequantise_kernel<<<dim3(blocks), dim3(kRowsPerBlock * 64), 0, st>>>(
        slot, n_rows, q_codes, q_scale, static_cast<const uint16_t*>(f_pool), sh, static_cast<uint16_t*>(out), ld_out);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
