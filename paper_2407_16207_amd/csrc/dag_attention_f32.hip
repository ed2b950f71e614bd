// fp32 DAG-masked attention (paper Sections 4.1 / 5.4): the small-shape, full-precision variant.
//
// One wavefront per (packed node, query head).  Lane l scores keys l, l+64, ... of the node's visible set
// (all prefix rows, then the draft rows whose mask bit is set), keeping its own running (max, sum, output);
// the 64 partial states are merged with wave shuffles at the end.  Plain FMA arithmetic, no matrix cores:
// this path exists for fp32 inputs and tight tolerances, the bf16 path is the fast one.
#include "gsd_internal.h"

namespace gsd {

template <int D>
__global__ __launch_bounds__(256) void dag_attention_f32_kernel(
    int32_t batch, int32_t max_nodes, int32_t total_rows, int32_t num_q_heads, int32_t group, int32_t words_per_row, float scale,
    const float *__restrict__ q, float *__restrict__ o, float *__restrict__ lse, const float *__restrict__ k,
    const float *__restrict__ v, const int64_t *__restrict__ kv_offsets, const int32_t *__restrict__ prefix_lens,
    const int32_t *__restrict__ node_offsets, const uint64_t *__restrict__ mask, int64_t q_ts, int64_t q_hs,
    int64_t o_ts, int64_t o_hs, int64_t kv_ts, int64_t kv_hs) {
    const int lane = threadIdx.x & 63;
    const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);     // row = t * Hq + h
    if (row >= total_rows) return;                                        // whole wave leaves together
    const int32_t t = int32_t(row / num_q_heads);
    const int32_t h = int32_t(row - int64_t(t) * num_q_heads);
    const int32_t hk = h / group;

    // sequence of node t: the last b with node_offsets[b] <= t
    int b = 0;
    while (b + 1 < batch && node_offsets[b + 1] <= t) ++b;
    const int32_t n = min(node_offsets[b + 1] - node_offsets[b], max_nodes);
    const int32_t P = prefix_lens[b];
    const int64_t kv0 = kv_offsets[b];
    const uint64_t *mrow = mask + int64_t(t) * words_per_row;

    float qr[D];
    const float *qp = q + t * q_ts + h * q_hs;
#pragma unroll
    for (int d = 0; d < D; d += 4) {
        const float4 x = *reinterpret_cast<const float4 *>(qp + d);
        qr[d] = x.x * scale; qr[d + 1] = x.y * scale; qr[d + 2] = x.z * scale; qr[d + 3] = x.w * scale;
    }
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    float m = -1e30f, l = 0.f;

    const int32_t total = P + n;
    for (int32_t j = lane; j < total; j += 64) {
        if (j >= P) {
            const int32_t dj = j - P;
            if (!((mrow[dj >> 6] >> (dj & 63)) & 1)) continue;
        }
        const float *kp = k + (kv0 + j) * kv_ts + hk * kv_hs;
        const float *vp = v + (kv0 + j) * kv_ts + hk * kv_hs;
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 x = *reinterpret_cast<const float4 *>(kp + d);
            s = fmaf(qr[d], x.x, s); s = fmaf(qr[d + 1], x.y, s);
            s = fmaf(qr[d + 2], x.z, s); s = fmaf(qr[d + 3], x.w, s);
        }
        const float m_new = fmaxf(m, s);
        const float alpha = __expf(m - m_new);
        const float p = __expf(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 x = *reinterpret_cast<const float4 *>(vp + d);
            acc[d] = fmaf(acc[d], alpha, p * x.x); acc[d + 1] = fmaf(acc[d + 1], alpha, p * x.y);
            acc[d + 2] = fmaf(acc[d + 2], alpha, p * x.z); acc[d + 3] = fmaf(acc[d + 3], alpha, p * x.w);
        }
        m = m_new;
    }

    // merge the 64 lane states
    float m_all = m;
    for (int off = 32; off > 0; off >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, off, 64));
    const float w = __expf(m - m_all);          // lanes that saw nothing: l == 0, acc == 0
    l *= w;
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off, 64);
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    float *op = o + t * o_ts + h * o_hs;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = acc[d] * w;
        for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
        if (lane == (d & 63)) op[d] = x * inv;
    }
    if (lse && lane == 0) lse[row] = (l > 0.f) ? m_all + __logf(l) : -__builtin_inff();
}

hipError_t launch_attention_f32(const gsd_attn_desc &d, hipStream_t stream) {
    const int64_t rows = int64_t(d.total_nodes) * d.num_q_heads;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    const int group = d.num_q_heads / d.num_kv_heads;
#define GSD_F32_ARGS                                                                                            \
    d.batch, d.max_nodes, (int32_t)rows, d.num_q_heads, group, d.words_per_row, d.softmax_scale, (const float *)d.q,         \
        (float *)d.o, d.lse, (const float *)d.k, (const float *)d.v, d.kv_offsets, d.prefix_lens,              \
        d.node_offsets, d.mask, d.q_token_stride, d.q_head_stride, d.o_token_stride, d.o_head_stride,          \
        d.kv_token_stride, d.kv_head_stride
    if (d.head_dim == 64)
        hipLaunchKernelGGL(dag_attention_f32_kernel<64>, grid, block, 0, stream, GSD_F32_ARGS);
    else
        hipLaunchKernelGGL(dag_attention_f32_kernel<128>, grid, block, 0, stream, GSD_F32_ARGS);
#undef GSD_F32_ARGS
    return hipGetLastError();
}

}  // namespace gsd
