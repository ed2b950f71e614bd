// Per-node vocabulary argmax of the verifier logits: the token the LLM itself would generate after each
// node (paper Section 3, deterministic verification).  Pure HBM streaming: one work-group per logits row,
// 16-byte loads, a (value, index) pair per lane, wave shuffles and one LDS hop to reduce.  The lowest index
// wins ties exactly (values are compared as stored); NaN never wins; an all-NaN row gives 0.
// With STATS the same sweep also carries the softmax normaliser of the row (running max and sum of exp(x - max),
// what non-deterministic verification needs, Section 3), so that both cost one pass over the logits.
#include "gsd_internal.h"

namespace gsd {

struct Best {
    float val;
    int32_t idx;   // INT32_MAX = nothing seen yet
};

__device__ __forceinline__ void consider(Best &b, float x, int32_t idx) {
    // elements are offered in ascending index order within a lane, so strict > keeps the first occurrence;
    // the equality arm only matters for the -inf start value.
    if (x > b.val || (x == b.val && idx < b.idx)) {
        b.val = x;
        b.idx = idx;
    }
}

__device__ __forceinline__ Best merge(Best a, Best o) {
    if (o.val > a.val || (o.val == a.val && o.idx < a.idx)) return o;
    return a;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// (m, s) <- merge of two partial softmax states: s counts exp(x - m)
__device__ __forceinline__ void merge_softmax_state(float &m, float &s, float m2, float s2) {
    const float mm = fmaxf(m, m2);
    if (mm == -__builtin_inff()) {          // both empty (or all -inf so far)
        m = mm;
        s = 0.f;
        return;
    }
    s = s * __expf(m - mm) + s2 * __expf(m2 - mm);
    m = mm;
}

template <int THREADS, bool BF16, bool NT, bool STATS>
__global__ __launch_bounds__(THREADS) void node_argmax_kernel(int32_t vocab, const void *__restrict__ logits,
                                                              int64_t row_stride, int32_t *__restrict__ pred,
                                                              float *__restrict__ row_max,
                                                              float *__restrict__ row_sumexp) {
    constexpr int ELT = BF16 ? 2 : 4;
    constexpr int PER_VEC = 16 / ELT;
    const int64_t row = blockIdx.x;
    const char *row_ptr = reinterpret_cast<const char *>(logits) + row * row_stride * ELT;
    Best best{-__builtin_inff(), 0x7fffffff};

    // scalar head up to the first 16-byte boundary, vector body, scalar tail
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row_ptr);
    int head = int(((16 - (addr & 15)) & 15) / ELT);
    if (head > vocab) head = vocab;
    const int nvec = (vocab - head) / PER_VEC;
    const int tail_start = head + nvec * PER_VEC;

    auto scalar_at = [&](int32_t i) -> float {
        if (BF16) return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t *>(row_ptr)[i]) << 16);
        return reinterpret_cast<const float *>(row_ptr)[i];
    };
    // softmax state of this lane (STATS): a batch of values joins it with one rescale
    float sm_m = -__builtin_inff(), sm_s = 0.f;
    auto add_batch = [&](const float *x, int cnt, float bm) {          // bm: max of the batch
        if (bm == -__builtin_inff()) return;
        const float mm = fmaxf(sm_m, bm);
        float add = 0.f;
        for (int j = 0; j < cnt; ++j) add += __expf(x[j] - mm);
        sm_s = sm_s * __expf(sm_m - mm) + add;
        sm_m = mm;
    };
    if (int(threadIdx.x) < head) {
        const float x = scalar_at(threadIdx.x);
        consider(best, x, threadIdx.x);
        if (STATS) add_batch(&x, 1, fmaxf(x, -__builtin_inff()));
    }

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *vec = reinterpret_cast<const u32x4 *>(row_ptr + size_t(head) * ELT);
    // Body: a lane only tracks the largest value and the 16-byte chunk it came from (one max tree and one compare
    // per chunk instead of a compare-and-select per element; the loads, not the ALU, should set the pace), and
    // looks the element up in that chunk afterwards.  Chunks come in ascending order, so a strict > keeps the
    // first chunk that holds the lane's maximum; NaN loses every v_max and every compare.
    float body_max = -__builtin_inff();
    int body_chunk = -1;
    u32x4 body_words = {0, 0, 0, 0};
    auto chunk_values = [&](const u32x4 w, float (&x)[PER_VEC]) {
        if (BF16) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[2 * j] = bf16_lo(w[j]);
                x[2 * j + 1] = bf16_hi(w[j]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(w[j]);
        }
    };
    // kBatch loads are issued before the first of them is looked at: with one load per lane in flight the row would
    // stream at the pace of memory latency (a wave has 1 KB on its way), not of memory bandwidth.  A slot past the end
    // of the row reads the last chunk again and is ignored.
    constexpr int kBatch = 8;
    for (int c0 = threadIdx.x; c0 < nvec; c0 += THREADS * kBatch) {
        u32x4 w[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int c = min(c0 + u * THREADS, nvec - 1);
            w[u] = NT ? __builtin_nontemporal_load(vec + c) : vec[c];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int c = c0 + u * THREADS;
            if (c >= nvec) break;
            float x[PER_VEC];
            chunk_values(w[u], x);
            float m = x[0];
#pragma unroll
            for (int j = 1; j < PER_VEC; ++j) m = fmaxf(m, x[j]);
            // the first chunk with any non-NaN value is taken even if that value is -inf (lowest index of an all -inf row)
            if (m > body_max || (body_chunk < 0 && m == body_max)) {
                body_max = m;
                body_chunk = c;
                body_words = w[u];   // kept in registers: fetching the chunk again at the end is a memory round trip per row
            }
            if (STATS) add_batch(x, PER_VEC, fmaxf(m, -__builtin_inff()));
        }
    }
    if (body_chunk >= 0) {
        float x[PER_VEC];
        chunk_values(body_words, x);
#pragma unroll
        for (int j = PER_VEC - 1; j >= 0; --j)
            if (x[j] == body_max) consider(best, x[j], head + body_chunk * PER_VEC + j);
    }
    {
        const int i = tail_start + threadIdx.x;
        if (i < vocab) {
            const float x = scalar_at(i);
            consider(best, x, i);
            if (STATS) add_batch(&x, 1, fmaxf(x, -__builtin_inff()));
        }
    }

    for (int off = 32; off > 0; off >>= 1) {
        Best o;
        o.val = __shfl_xor(best.val, off, 64);
        o.idx = __shfl_xor(best.idx, off, 64);
        best = merge(best, o);
        if (STATS) {
            const float m2 = __shfl_xor(sm_m, off, 64), s2 = __shfl_xor(sm_s, off, 64);
            merge_softmax_state(sm_m, sm_s, m2, s2);
        }
    }
    __shared__ float s_val[THREADS / 64];
    __shared__ int32_t s_idx[THREADS / 64];
    __shared__ float s_m[THREADS / 64], s_s[THREADS / 64];
    if ((threadIdx.x & 63) == 0) {
        s_val[threadIdx.x >> 6] = best.val;
        s_idx[threadIdx.x >> 6] = best.idx;
        if (STATS) {
            s_m[threadIdx.x >> 6] = sm_m;
            s_s[threadIdx.x >> 6] = sm_s;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        Best r{s_val[0], s_idx[0]};
        for (int w = 1; w < THREADS / 64; ++w) r = merge(r, Best{s_val[w], s_idx[w]});
        pred[row] = (r.idx == 0x7fffffff) ? 0 : r.idx;
        if (STATS) {
            float M = s_m[0], S = s_s[0];
            for (int w = 1; w < THREADS / 64; ++w) merge_softmax_state(M, S, s_m[w], s_s[w]);
            row_max[row] = M;
            row_sumexp[row] = S;
        }
    }
}

hipError_t launch_node_argmax(int32_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                              int32_t *pred, float *row_max, float *row_sumexp, hipStream_t stream) {
    // Few rows: large work-groups so each row still has many loads in flight.
    const bool big = rows < 1024;
    // Measured on this chip with 32000-entry bf16 rows: logits that fit the 256 MB last-level cache stream faster
    // with non-temporal loads (131 MB: 5.27 against 4.93 TB/s), larger ones with ordinary loads (1 GB: 5.25 against
    // 4.89 TB/s).
    const bool nt = double(rows) * double(vocab) * (dtype == GSD_BF16 ? 2 : 4) < 192e6;
    const bool stats = row_max != nullptr;
#define GSD_ARGMAX_LAUNCH(THREADS, BF16, NT, STATS)                                                                 \
    hipLaunchKernelGGL((node_argmax_kernel<THREADS, BF16, NT, STATS>), dim3(rows), dim3(THREADS), 0, stream, vocab,  \
                       logits, row_stride, pred, row_max, row_sumexp)
#define GSD_ARGMAX_PICK(BF16, STATS)                                                                                \
    do {                                                                                                            \
        if (big) { if (nt) GSD_ARGMAX_LAUNCH(1024, BF16, true, STATS); else GSD_ARGMAX_LAUNCH(1024, BF16, false, STATS); } \
        else { if (nt) GSD_ARGMAX_LAUNCH(256, BF16, true, STATS); else GSD_ARGMAX_LAUNCH(256, BF16, false, STATS); }  \
    } while (0)
    if (dtype == GSD_BF16) {
        if (stats) GSD_ARGMAX_PICK(true, true); else GSD_ARGMAX_PICK(true, false);
    } else {
        if (stats) GSD_ARGMAX_PICK(false, true); else GSD_ARGMAX_PICK(false, false);
    }
#undef GSD_ARGMAX_PICK
#undef GSD_ARGMAX_LAUNCH
    return hipGetLastError();
}

}  // namespace gsd
