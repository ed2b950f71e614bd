// Non-deterministic verification (paper Section 3: the i-th drafted token is accepted with probability
// min(1, p/q), the first rejection discards the rest of the hypothesis and the LLM regenerates that token;
// Section 6.4: the setting on token graphs).  Three kernels:
//
//   softmax_stats_kernel    one pass over a logits row: running (max, sum of exp(x - max)) per lane, merged across
//                           the work-group: the normaliser of the LLM's distribution after every node.  HBM-bound,
//                           same traffic as the argmax pass of deterministic verification.
//   accept_stochastic_kernel one work-group per sequence: every edge r -> i is tested once,
//                               accept_u[i] * draft_prob[i] < p_r(token_i)      (<=> u < min(1, p/q) for u < 1)
//                           with p_r(token_i) = exp(logit - max_r) / sum_r gathered from the row of r, then the same
//                           relaxation, end-node choice and back-walk as the deterministic kernel.
//   resample_kernel         one work-group per sequence: the regenerated token, drawn by inverse CDF from
//                           max(p - q, 0) at the end of the accepted path (from p if that node has no children or the
//                           residual is empty).  Every thread owns a contiguous slice of the vocabulary, slice sums
//                           are scanned in thread order, the owning thread walks its slice: one fixed summation order.
//                           (resample_held_kernel: the same with the slices kept in registers, where they fit.)
#include "gsd_internal.h"

namespace gsd {

__device__ __forceinline__ float load_logit(const void *base, int64_t elem, int dtype) {
    if (dtype == GSD_BF16) return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t *>(base)[elem]) << 16);
    return reinterpret_cast<const float *>(base)[elem];
}

// (m, s) <- merge of two partial softmax states: s counts exp(x - m)
__device__ __forceinline__ void merge_state(float &m, float &s, float m2, float s2) {
    const float mm = fmaxf(m, m2);
    if (mm == -__builtin_inff()) {          // both empty (or all -inf so far)
        m = mm;
        s = 0.f;
        return;
    }
    s = s * __expf(m - mm) + s2 * __expf(m2 - mm);
    m = mm;
}

template <int THREADS, bool BF16>
__global__ __launch_bounds__(THREADS) void softmax_stats_kernel(int32_t vocab, const void *__restrict__ logits,
                                                                int64_t row_stride, float *__restrict__ row_max,
                                                                float *__restrict__ row_sumexp, int64_t rows_first,
                                                                const void *__restrict__ logits_after) {
    constexpr int ELT = BF16 ? 2 : 4;
    constexpr int PER_VEC = 16 / ELT;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int64_t row = blockIdx.x;                      // rows beyond the first buffer's come from the second
    const char *row_ptr = row < rows_first
                              ? reinterpret_cast<const char *>(logits) + row * row_stride * ELT
                              : reinterpret_cast<const char *>(logits_after) + (row - rows_first) * row_stride * ELT;
    float m = -__builtin_inff(), s = 0.f;
    // a batch of values joins the running state with one rescale: max of the batch first, then its exponentials
    auto add_batch = [&](const float *x, int cnt) {
        float bm = -__builtin_inff();
        for (int j = 0; j < cnt; ++j) bm = fmaxf(bm, x[j]);
        if (bm == -__builtin_inff()) return;
        const float mm = fmaxf(m, bm);
        float add = 0.f;
        for (int j = 0; j < cnt; ++j) add += __expf(x[j] - mm);
        s = s * __expf(m - mm) + add;
        m = mm;
    };
    // scalar head up to the first 16-byte boundary, 16-byte body, scalar tail
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row_ptr);
    int head = int(((16 - (addr & 15)) & 15) / ELT);
    if (head > vocab) head = vocab;
    const int nvec = (vocab - head) / PER_VEC;
    const int tail_start = head + nvec * PER_VEC;
    auto scalar_at = [&](int32_t i) -> float {
        if (BF16) return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t *>(row_ptr)[i]) << 16);
        return reinterpret_cast<const float *>(row_ptr)[i];
    };
    if (int(threadIdx.x) < head) {
        const float x = scalar_at(threadIdx.x);
        add_batch(&x, 1);
    }
    const u32x4 *vec = reinterpret_cast<const u32x4 *>(row_ptr + size_t(head) * ELT);
    // kBatch loads are issued before the first of them is looked at (one load per lane in flight streams at the pace of
    // memory latency, not bandwidth); a slot past the end of the row reads the last chunk again and is ignored
    constexpr int kBatch = 8;
    for (int c0 = threadIdx.x; c0 < nvec; c0 += THREADS * kBatch) {
        u32x4 w[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) w[u] = __builtin_nontemporal_load(vec + min(c0 + u * THREADS, nvec - 1));
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (c0 + u * THREADS >= nvec) break;
            float x[PER_VEC];
            if (BF16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    x[2 * j] = __uint_as_float(w[u][j] << 16);
                    x[2 * j + 1] = __uint_as_float(w[u][j] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(w[u][j]);
            }
            add_batch(x, PER_VEC);
        }
    }
    {
        const int i = tail_start + threadIdx.x;
        if (i < vocab) {
            const float x = scalar_at(i);
            add_batch(&x, 1);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, 64), s2 = __shfl_xor(s, off, 64);
        merge_state(m, s, m2, s2);
    }
    __shared__ float sm[THREADS / 64], ss[THREADS / 64];
    if ((threadIdx.x & 63) == 0) {
        sm[threadIdx.x >> 6] = m;
        ss[threadIdx.x >> 6] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = sm[0], S = ss[0];
        for (int w = 1; w < THREADS / 64; ++w) merge_state(M, S, sm[w], ss[w]);
        row_max[row] = M;
        row_sumexp[row] = S;
    }
}

hipError_t launch_softmax_stats(int64_t rows, int32_t vocab, int dtype, const void *logits, int64_t row_stride,
                                float *row_max, float *row_sumexp, hipStream_t stream, int64_t rows_after,
                                const void *logits_after) {
    const dim3 grid((unsigned)(rows + rows_after));
    if (dtype == GSD_BF16)
        hipLaunchKernelGGL((softmax_stats_kernel<256, true>), grid, dim3(256), 0, stream, vocab, logits, row_stride,
                           row_max, row_sumexp, rows, logits_after);
    else
        hipLaunchKernelGGL((softmax_stats_kernel<256, false>), grid, dim3(256), 0, stream, vocab, logits, row_stride,
                           row_max, row_sumexp, rows, logits_after);
    return hipGetLastError();
}

constexpr int kStochThreads = 512;

__global__ __launch_bounds__(kStochThreads) void accept_stochastic_kernel(const gsd_stochastic_desc d) {
    __shared__ int32_t L[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t path_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ int32_t back_s[GSD_MAX_NODES_PER_SEQ];
    __shared__ uint32_t wave_best[kStochThreads / 64];
    __shared__ int32_t len_s;
    static_assert(kStochThreads >= GSD_MAX_NODES_PER_SEQ, "one thread per node");

    const int b = blockIdx.x;
    const int64_t base = d.node_offsets[b];
    int n = d.node_offsets[b + 1] - d.node_offsets[b];
    if (n > d.max_nodes) n = d.max_nodes;
    if (n < 0) n = 0;
    const float *root_max = d.row_max + d.total_nodes, *root_sum = d.row_sumexp + d.total_nodes;

    // One thread per node.  Whether an edge passes never changes, so every node tests its own parent edges once
    // (its coin against the LLM's probability of its token after that parent) and keeps the first four that pass
    // in registers; the loads of the four tests are issued together, with clamped indices instead of branches.
    constexpr int kRegParents = 4;
    const int i = threadIdx.x;
    const bool active = i < n;
    int par[kRegParents];          // parent id of a passing edge; -1 = root; -2 = no such edge, or it did not pass
#pragma unroll
    for (int x = 0; x < kRegParents; ++x) par[x] = -2;
    int32_t e_lo = 0, e_hi = 0;    // this node's slice of parent_idx
    int32_t tok = 0;
    bool tok_ok = false;           // a token outside the vocabulary is never accepted
    float coin = 0.f;              // accept_u * draft_prob: the edge passes iff coin < p_r(tok)
    // the LLM's probability of this node's token after parent r (a well-formed parent, -1 = the root)
    auto prob_after = [&](int r) -> float {
        const void *rows = r == -1 ? d.root_logits : d.logits;
        const int64_t row = r == -1 ? int64_t(b) : base + r;
        const float mx = r == -1 ? root_max[b] : d.row_max[base + r];
        const float sm = r == -1 ? root_sum[b] : d.row_sumexp[base + r];
        return __expf(load_logit(rows, row * d.row_stride + tok, d.dtype) - mx) / sm;
    };
    if (active) {
        e_lo = d.parent_offsets[base + i];
        e_hi = d.parent_offsets[base + i + 1];
        tok = d.tokens[base + i];
        coin = d.accept_u[base + i] * d.draft_prob[base + i];
        tok_ok = tok >= 0 && tok < d.vocab;
        if (!tok_ok) tok = 0;                                  // keeps the gathers below in bounds
        if (e_hi > e_lo) {
            int r[kRegParents];
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) r[x] = d.parent_idx[min(e_lo + x, e_hi - 1)];
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) {
                const bool wf = e_lo + x < e_hi && r[x] >= -1 && r[x] < i;
                const float pr = prob_after(wf ? r[x] : -1);
                if (wf && tok_ok && coin < pr) par[x] = r[x];
            }
        }
        L[i] = -1;
    }
    const bool more = active && e_hi - e_lo > kRegParents;     // rare: a node with more than four parents
    auto passes = [&](int r) -> bool { return r >= -1 && r < i && tok_ok && coin < prob_after(r); };
    __syncthreads();

    int32_t mine = -1;             // L[i]
    for (int sweep = 0; sweep <= n; ++sweep) {
        int changed = 0;
        if (active) {
            int32_t best = mine;
#pragma unroll
            for (int x = 0; x < kRegParents; ++x) {
                const int32_t l = L[par[x] >= 0 ? par[x] : i];
                const int32_t lr = par[x] >= 0 ? l : (par[x] == -1 ? 0 : -1);
                if (lr >= 0 && lr + 1 > best) best = lr + 1;
            }
            if (more) {
                for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                    const int r = d.parent_idx[e];
                    if (!passes(r)) continue;
                    const int32_t lr = (r == -1) ? 0 : L[r];
                    if (lr >= 0 && lr + 1 > best) best = lr + 1;
                }
            }
            if (best != mine) {
                mine = best;
                L[i] = best;
                changed = 1;
            }
        }
        if (!__syncthreads_or(changed)) break;
    }

    // back pointer of every accepted node: the smallest-id passing parent that ends a path one node shorter
    if (active && mine > 0) {
        int32_t chosen = 0x7fffffff;
#pragma unroll
        for (int x = 0; x < kRegParents; ++x) {
            const int32_t l = L[par[x] >= 0 ? par[x] : i];
            const int32_t lr = par[x] >= 0 ? l : (par[x] == -1 ? 0 : -1);
            if (lr == mine - 1 && par[x] < chosen) chosen = par[x];
        }
        if (more) {
            for (int e = e_lo + kRegParents; e < e_hi; ++e) {
                const int r = d.parent_idx[e];
                if (!passes(r)) continue;
                const int32_t lr = (r == -1) ? 0 : L[r];
                if (lr == mine - 1 && r < chosen) chosen = r;
            }
        }
        back_s[i] = chosen;
    }

    uint32_t key = 0;                                    // largest L, then smallest id
    if (active && mine > 0) key = uint32_t(mine) * 1024u + uint32_t(1023 - i);
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t other = __shfl_xor(key, off, 64);
        key = other > key ? other : key;
    }
    if ((threadIdx.x & 63) == 0) wave_best[threadIdx.x >> 6] = key;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t k = 0;
        for (int w = 0; w < kStochThreads / 64; ++w) k = wave_best[w] > k ? wave_best[w] : k;
        const int32_t len = int32_t(k / 1024u);
        int32_t v = (len > 0) ? int32_t(1023u - (k % 1024u)) : -1;
        len_s = len;
        d.accept_len[b] = len;
        d.end_node[b] = v;
        for (int pos = len - 1; pos >= 0 && v >= 0 && v < n; --pos) {   // L drops by one per step: the root's child sits at pos 0
            path_s[pos] = v;
            v = back_s[v];
        }
    }
    __syncthreads();
    const int32_t len = len_s;
    int32_t *out = d.accept_path + int64_t(b) * d.max_nodes;
    for (int x = threadIdx.x; x < d.max_nodes; x += kStochThreads) out[x] = (x < len) ? path_s[x] : -1;
}

constexpr int kResampleThreads = 1024;

__global__ __launch_bounds__(kResampleThreads) void resample_kernel(const gsd_stochastic_desc d) {
    __shared__ float red_m[kResampleThreads / 64], red_s[kResampleThreads / 64];
    __shared__ float part[kResampleThreads];
    __shared__ float stat[4];
    __shared__ int has_child_s, pick_s;

    const int b = blockIdx.x;
    const int64_t base = d.node_offsets[b];
    int n = d.node_offsets[b + 1] - d.node_offsets[b];
    if (n > d.max_nodes) n = d.max_nodes;
    if (n < 0) n = 0;
    const int end = d.end_node[b];
    const int V = d.vocab;

    // does the end node (or the root) have children ?
    if (threadIdx.x == 0) {
        has_child_s = 0;
        pick_s = -1;
    }
    __syncthreads();
    const int32_t e0 = d.parent_offsets[base], e1 = d.parent_offsets[base + n];
    int mine = 0;
    for (int e = e0 + threadIdx.x; e < e1; e += kResampleThreads) mine |= (d.parent_idx[e] == end);
    if (mine) has_child_s = 1;

    const void *p_row = end < 0 ? d.root_logits : d.logits;
    const void *q_row = end < 0 ? d.root_draft_logits : d.draft_logits;
    const int64_t row_off = (end < 0 ? int64_t(b) : base + end) * d.row_stride;
    const float p_max = end < 0 ? d.row_max[d.total_nodes + b] : d.row_max[base + end];
    const float p_sum = end < 0 ? d.row_sumexp[d.total_nodes + b] : d.row_sumexp[base + end];

    // the draft row's own (max, sum)
    float m = -__builtin_inff(), s = 0.f;
    for (int x = threadIdx.x; x < V; x += kResampleThreads) merge_state(m, s, load_logit(q_row, row_off + x, d.dtype), 1.f);
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, 64), s2 = __shfl_xor(s, off, 64);
        merge_state(m, s, m2, s2);
    }
    if ((threadIdx.x & 63) == 0) {
        red_m[threadIdx.x >> 6] = m;
        red_s[threadIdx.x >> 6] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = red_m[0], S = red_s[0];
        for (int w = 1; w < kResampleThreads / 64; ++w) merge_state(M, S, red_m[w], red_s[w]);
        stat[0] = M;
        stat[1] = S;
    }
    __syncthreads();
    const float q_max = stat[0], q_sum = stat[1];
    const bool use_residual = has_child_s != 0;

    // contiguous slice of the vocabulary per thread
    const int per = (V + kResampleThreads - 1) / kResampleThreads;
    const int x0 = threadIdx.x * per, x1 = min(V, x0 + per);
    auto weight = [&](int x, bool residual) -> float {
        const float p = __expf(load_logit(p_row, row_off + x, d.dtype) - p_max) / p_sum;
        if (!residual) return p;
        const float q = __expf(load_logit(q_row, row_off + x, d.dtype) - q_max) / q_sum;
        return fmaxf(p - q, 0.f);
    };
    // The weights of this thread's slice, in ascending token order, handed to f(x, w) until f returns true.  A slice
    // is contiguous in memory, so when it starts on a 16-byte boundary it is fetched 16 bytes at a time (one load
    // per 8 bf16 / 4 fp32 values instead of one per value: the lanes of a wave are a slice apart, so every load
    // instruction touches 64 cache lines whatever its width); same values, same order either way.
    const int elt = d.dtype == GSD_BF16 ? 2 : 4;
    const int per_vec = 16 / elt;
    const bool vec_ok = (per * elt) % 16 == 0 &&
                        (reinterpret_cast<uintptr_t>(p_row) + uintptr_t(row_off) * elt) % 16 == 0 &&
                        (reinterpret_cast<uintptr_t>(q_row) + uintptr_t(row_off) * elt) % 16 == 0;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    auto unpack = [&](const u32x4 v, float (&out)[8]) {
        if (d.dtype == GSD_BF16) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                out[2 * j] = __uint_as_float(v[j] << 16);
                out[2 * j + 1] = __uint_as_float(v[j] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = __uint_as_float(v[j]);
        }
    };
    auto for_each_weight = [&](bool residual, auto &&f) {
        int x = x0;
        if (vec_ok) {
            for (; x + per_vec <= x1; x += per_vec) {
                float lp[8], lq[8];
                unpack(*reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(p_row) + (row_off + x) * elt), lp);
                if (residual)
                    unpack(*reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(q_row) + (row_off + x) * elt), lq);
                for (int j = 0; j < per_vec; ++j) {
                    const float pp = __expf(lp[j] - p_max) / p_sum;
                    const float w = residual ? fmaxf(pp - __expf(lq[j] - q_max) / q_sum, 0.f) : pp;
                    if (f(x + j, w)) return;
                }
            }
        }
        for (; x < x1; ++x)
            if (f(x, weight(x, residual))) return;
    };
    // total weight (thread-ordered scan in LDS, fixed order), falling back to p when the residual is empty
    auto scan = [&](bool residual) -> float {
        float local = 0.f;
        for_each_weight(residual, [&](int, float w) {
            local += w;
            return false;
        });
        __syncthreads();
        part[threadIdx.x] = local;
        __syncthreads();
        for (int dd = 1; dd < kResampleThreads; dd <<= 1) {      // inclusive scan
            const float add = int(threadIdx.x) >= dd ? part[threadIdx.x - dd] : 0.f;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        return part[kResampleThreads - 1];
    };
    bool residual = use_residual;
    float total = scan(residual);
    if (residual && !(total > 0.f)) {
        residual = false;
        total = scan(false);
    }
    const float target = d.resample_u[b] * total;
    const float before = threadIdx.x > 0 ? part[threadIdx.x - 1] : 0.f;
    const float upto = part[threadIdx.x];
    // the owner of the target walks its slice; the smallest token whose cumulative weight exceeds the target
    if (before <= target && target < upto) {
        float run = before;
        int pick = -1;
        for_each_weight(residual, [&](int x, float w) {
            run += w;
            if (run > target) {
                pick = x;
                return true;
            }
            return false;
        });
        if (pick < 0) {                                     // rounding inside the slice: its last token with weight
            for (int x = x1 - 1; x >= x0; --x)
                if (weight(x, residual) > 0.f) {
                    pick = x;
                    break;
                }
        }
        pick_s = pick;
    }
    __syncthreads();
    if (pick_s < 0 && threadIdx.x == 0) {                    // target == total by rounding: the last token with weight
        int pick = 0;
        for (int x = V - 1; x >= 0; --x)
            if (weight(x, residual) > 0.f) {
                pick = x;
                break;
            }
        pick_s = pick;
    }
    __syncthreads();
    if (threadIdx.x == 0) d.bonus_token[b] = pick_s;
}

// The same draw for rows whose per-thread slice fits registers (the launcher checks: the slice is a whole number of
// 16-byte runs, at most kHeld values, rows start on 16-byte boundaries, the vocabulary ends on one): a thread fetches
// its slice of both rows once, all loads in flight together, and every later step works from those registers: the
// draft row's normaliser, the slice's weight sum, and (for the one thread that owns the target) the walk.  Scans go
// through wave shuffles and one LDS hop instead of a log-step LDS scan; the order of every sum is fixed.
constexpr int kHeld = 32;

template <bool BF16>
__global__ __launch_bounds__(kResampleThreads) void resample_held_kernel(const gsd_stochastic_desc d) {
    constexpr int ELT = BF16 ? 2 : 4;
    constexpr int PER_VEC = 16 / ELT;
    constexpr int KV = kHeld / PER_VEC;
    constexpr int kWaves = kResampleThreads / 64;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    __shared__ float red_m[kWaves], red_s[kWaves], wave_sum[2][kWaves];
    __shared__ int pick_s;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int b = blockIdx.x;
    const int64_t base = d.node_offsets[b];
    int n = d.node_offsets[b + 1] - d.node_offsets[b];
    if (n > d.max_nodes) n = d.max_nodes;
    if (n < 0) n = 0;
    const int end = d.end_node[b];
    const int V = d.vocab;
    if (t == 0) pick_s = -1;

    const int64_t row_off = (end < 0 ? int64_t(b) : base + end) * d.row_stride;
    const char *p_ptr = reinterpret_cast<const char *>(end < 0 ? d.root_logits : d.logits) + row_off * ELT;
    const char *q_ptr = reinterpret_cast<const char *>(end < 0 ? d.root_draft_logits : d.draft_logits) + row_off * ELT;
    const int per = (V + kResampleThreads - 1) / kResampleThreads;
    const int x0 = t * per;
    const int nvec = x0 < V ? min(per, V - x0) / PER_VEC : 0;     // whole 16-byte runs: the vocabulary ends on one
    u32x4 raw_p[KV], raw_q[KV];
#pragma unroll
    for (int j = 0; j < KV; ++j) {                                // a run this thread does not have reads the row's first
        const int64_t off = (j < nvec ? int64_t(x0) + j * PER_VEC : 0) * ELT;
        raw_q[j] = *reinterpret_cast<const u32x4 *>(q_ptr + off);
        raw_p[j] = *reinterpret_cast<const u32x4 *>(p_ptr + off);
    }
    const float p_max = end < 0 ? d.row_max[d.total_nodes + b] : d.row_max[base + end];
    const float p_sum = end < 0 ? d.row_sumexp[d.total_nodes + b] : d.row_sumexp[base + end];
    // does the end node (or the root) have children ?
    const int32_t e0 = d.parent_offsets[base], e1 = d.parent_offsets[base + n];
    int mine = 0;
    for (int e = e0 + t; e < e1; e += kResampleThreads) mine |= (d.parent_idx[e] == end);

    auto value = [&](const u32x4 v, int e) -> float {
        if (BF16) return (e & 1) ? __uint_as_float(v[e >> 1] & 0xffff0000u) : __uint_as_float(v[e >> 1] << 16);
        return __uint_as_float(v[e]);
    };
    // the draft row's own (max, sum)
    float m = -__builtin_inff(), sum = 0.f;
#pragma unroll
    for (int j = 0; j < KV; ++j)
        if (j < nvec) {
#pragma unroll
            for (int e = 0; e < PER_VEC; ++e) m = fmaxf(m, value(raw_q[j], e));
        }
    if (m > -__builtin_inff()) {
#pragma unroll
        for (int j = 0; j < KV; ++j)
            if (j < nvec) {
#pragma unroll
                for (int e = 0; e < PER_VEC; ++e) sum += __expf(value(raw_q[j], e) - m);
            }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, 64), s2 = __shfl_xor(sum, off, 64);
        merge_state(m, sum, m2, s2);
    }
    if (lane == 0) {
        red_m[wave] = m;
        red_s[wave] = sum;
    }
    const bool use_residual = __syncthreads_or(mine) != 0;
    float q_max = red_m[0], q_sum = red_s[0];
    for (int w = 1; w < kWaves; ++w) merge_state(q_max, q_sum, red_m[w], red_s[w]);

    const float p_scale = 1.f / p_sum, q_scale = 1.f / q_sum;     // one division per row instead of one per token
    auto weight_of = [&](float lp, float lq, bool residual) -> float {
        const float pp = __expf(lp - p_max) * p_scale;
        return residual ? fmaxf(pp - __expf(lq - q_max) * q_scale, 0.f) : pp;
    };
    // the cumulative weight before this thread's slice and up to its end: the slice in ascending token order, the
    // wave in lane order, the waves in their order
    float before = 0.f, upto = 0.f, total = 0.f;
    auto scan = [&](bool residual, int turn) {
        float local = 0.f;
#pragma unroll
        for (int j = 0; j < KV; ++j)
            if (j < nvec) {
#pragma unroll
                for (int e = 0; e < PER_VEC; ++e) local += weight_of(value(raw_p[j], e), value(raw_q[j], e), residual);
            }
        float incl = local;
#pragma unroll
        for (int dd = 1; dd < 64; dd <<= 1) {
            const float up = __shfl_up(incl, dd, 64);
            if (lane >= dd) incl += up;
        }
        const float left = __shfl_up(incl, 1, 64);
        if (lane == 63) wave_sum[turn][wave] = incl;
        __syncthreads();
        float run = 0.f, mine_base = 0.f;
        for (int w = 0; w < kWaves; ++w) {
            if (w == wave) mine_base = run;
            run += wave_sum[turn][w];
        }
        total = run;
        before = lane == 0 ? mine_base : mine_base + left;
        upto = mine_base + incl;
    };
    bool residual = use_residual;
    scan(residual, 0);
    if (residual && !(total > 0.f)) {                        // empty residual: draw from p
        residual = false;
        scan(false, 1);
    }
    const float target = d.resample_u[b] * total;
    // the owner of the target walks its slice; the smallest token whose cumulative weight exceeds the target
    if (before <= target && target < upto) {
        float run = before;
        int pick = -1, last = -1;
#pragma unroll
        for (int j = 0; j < KV; ++j)
            if (j < nvec) {
#pragma unroll
                for (int e = 0; e < PER_VEC; ++e) {
                    const float w = weight_of(value(raw_p[j], e), value(raw_q[j], e), residual);
                    run += w;
                    if (w > 0.f) last = x0 + j * PER_VEC + e;
                    if (pick < 0 && run > target) pick = x0 + j * PER_VEC + e;
                }
            }
        pick_s = pick >= 0 ? pick : last;                   // rounding inside the slice: its last token with weight
    }
    __syncthreads();
    if (pick_s < 0) {                                       // target == total by rounding: the last token with weight
        int last = -1;
#pragma unroll
        for (int j = 0; j < KV; ++j)
            if (j < nvec) {
#pragma unroll
                for (int e = 0; e < PER_VEC; ++e)
                    if (weight_of(value(raw_p[j], e), value(raw_q[j], e), residual) > 0.f) last = x0 + j * PER_VEC + e;
            }
        for (int off = 32; off > 0; off >>= 1) last = max(last, __shfl_xor(last, off, 64));
        __shared__ int wave_last[kWaves];
        if (lane == 0) wave_last[wave] = last;
        __syncthreads();
        if (t == 0) {
            int best = 0;
            for (int w = 0; w < kWaves; ++w) best = max(best, wave_last[w]);
            pick_s = best;
        }
        __syncthreads();
    }
    if (t == 0) d.bonus_token[b] = pick_s;
}

hipError_t launch_accept_stochastic(const gsd_stochastic_desc &d, hipStream_t stream) {
    // the node rows and, behind them, the root rows: one launch
    hipError_t err = launch_softmax_stats(d.total_nodes, d.vocab, d.dtype, d.logits, d.row_stride, d.row_max,
                                          d.row_sumexp, stream, d.batch, d.root_logits);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(accept_stochastic_kernel, dim3(d.batch), dim3(kStochThreads), 0, stream, d);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    // slices that fit registers: see resample_held_kernel
    const int elt = d.dtype == GSD_BF16 ? 2 : 4;
    const int per = (d.vocab + kResampleThreads - 1) / kResampleThreads;
    auto aligned = [&](const void *ptr) { return reinterpret_cast<uintptr_t>(ptr) % 16 == 0; };
    const bool held = per <= kHeld && (per * elt) % 16 == 0 && (int64_t(d.vocab) * elt) % 16 == 0 &&
                      (d.row_stride * elt) % 16 == 0 && aligned(d.logits) && aligned(d.root_logits) &&
                      aligned(d.draft_logits) && aligned(d.root_draft_logits);
    if (held && d.dtype == GSD_BF16)
        hipLaunchKernelGGL(resample_held_kernel<true>, dim3(d.batch), dim3(kResampleThreads), 0, stream, d);
    else if (held)
        hipLaunchKernelGGL(resample_held_kernel<false>, dim3(d.batch), dim3(kResampleThreads), 0, stream, d);
    else
        hipLaunchKernelGGL(resample_kernel, dim3(d.batch), dim3(kResampleThreads), 0, stream, d);
    return hipGetLastError();
}

}  // namespace gsd
