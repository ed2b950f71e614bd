// bf16 DAG-masked flash attention for gfx950 (paper Sections 4.1 / 5.4: one verifier pass over the flattened
// token graph; every draft node attends to the whole context and to its visible draft nodes).
//
// Shape of the work.  All G = Hq/Hkv query heads of a KV head share its K/V rows and (per node) the same mask
// row, so the (node, head) pairs of one (sequence, KV head) are packed into one row space r = node*G + g and
// cut into tiles of 128 rows; a work-group of 4 wavefronts owns one tile (32 rows per wave) and walks the KV
// axis in tiles of 64 keys: first the prefix tiles (no mask code at all, only the ragged last tile is
// bounded), then the draft tiles, one 64-bit mask word per row per tile; a draft tile whose word is zero for
// every row of the work-group is skipped outright.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  Scores are computed TRANSPOSED,
// S^T = K . Q^T, so that a lane owns one query row (column n = lane%32) and 16 keys per 32-key block: row
// max and row sum are in-lane loops plus one exchange with lane^32, and the running rescale factor is a
// per-lane scalar for the O^T = V^T . P^T accumulators, which have the same column ownership.  The S^T
// accumulator registers are converted to bf16 in place and fed straight back as the B operand of the second
// contraction: K rows are stored in LDS in the order that makes each lane's 8 consecutive accumulator
// registers 8 consecutive keys, and V is stored with adjacent key pairs interleaved per channel so that the
// A operand of the second contraction is four 32-bit LDS reads per lane.
//
// Small problems are split along the KV axis (gsd_attn_desc.num_splits); a split writes unnormalised fp32
// partials (O, running max, running sum) and a second kernel merges them in split order.
#include "gsd_internal.h"

namespace gsd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kRowsPerWG = 128;      // query rows (node, head pairs) per work-group
constexpr int kKeysPerTile = 64;     // keys per KV tile = one mask word
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMInit = -1e30f;     // finite stand-in for -inf as the running max

struct AttnParams {
    const __bf16 *q;
    __bf16 *o;
    float *lse;
    const __bf16 *k;
    const __bf16 *v;
    const int64_t *kv_offsets;
    const int32_t *prefix_lens;
    const int32_t *node_offsets;
    const uint64_t *mask;
    float *part_o;      // [splits][T][Hq][D] fp32 unnormalised
    float *part_ml;     // [splits][T][Hq][2]  (running max of raw scores, running sum)
    int64_t q_ts, q_hs, o_ts, o_hs, kv_ts, kv_hs;
    int32_t batch, total_nodes, max_nodes, num_q_heads, num_kv_heads, group, words_per_row;
    int32_t q_tiles;    // row tiles per (sequence, KV head)
    int32_t splits;
    int32_t total_wg;   // q_tiles * splits * batch * num_kv_heads
    int32_t wg_per_xcd; // ceil(total_wg / 8)
    float scale_log2e;  // softmax_scale * log2(e)
    float scale;
};

template <int D>
struct Lds {
    static constexpr int kKRowBytes = D * 2 + 16;                 // padded K row
    static constexpr int kKBytes = kKeysPerTile * kKRowBytes;
    static constexpr int kVRowBytes = D * 4;                      // one key PAIR x D channels, 4 bytes each
    static constexpr int kVBytes = (kKeysPerTile / 2) * kVRowBytes;
    static constexpr int kTotal = kKBytes + kVBytes;
};

// position of actual key row r (0..63) inside the LDS K tile: bits 2 and 3 of r swapped (see file comment)
__device__ __forceinline__ int k_lds_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

template <int D>
__global__ __launch_bounds__(kThreads, 2) void dag_attention_bf16_kernel(const AttnParams p) {
    constexpr int KS = D / 16;          // k-steps of the first contraction
    constexpr int MBD = D / 32;         // 32-channel blocks of the output
    constexpr int CHUNKS = D / 8;       // 16-byte chunks per K/V row
    constexpr int ROWS_PER_PASS = kThreads / CHUNKS;
    constexpr int K_PASSES = kKeysPerTile / ROWS_PER_PASS;
    constexpr int V_PASSES = (kKeysPerTile / 2) / ROWS_PER_PASS;
    using L = Lds<D>;
    __shared__ __attribute__((aligned(16))) char lds[L::kTotal];
    char *lds_k = lds;
    char *lds_v = lds + L::kKBytes;

    // ---- which piece of work: XCD-aware decode of the linear work-group id --------------------------------
    // Hardware deals consecutive work-group ids round-robin to the 8 XCDs; give every XCD a contiguous range
    // of logical ids so that the row tiles sharing one K/V stream run on one XCD and share its L2.
    const int hw = blockIdx.x;
    const int logical = (hw & 7) * p.wg_per_xcd + (hw >> 3);
    if (logical >= p.total_wg) return;
    const int qt = logical % p.q_tiles;
    const int rest = logical / p.q_tiles;
    const int split = rest % p.splits;
    const int group_id = rest / p.splits;          // b * Hkv + kvh
    const int b = group_id / p.num_kv_heads;
    const int kvh = group_id - b * p.num_kv_heads;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int half = lane >> 5;        // which 8-wide k group / which 4-row group of the accumulator
    const int col = lane & 31;         // query row inside the wave's 32

    const int32_t node_base = p.node_offsets[b];
    const int32_t n = min(p.node_offsets[b + 1] - node_base, p.max_nodes);   // never trust past the stated bound
    const int32_t P = p.prefix_lens[b];
    const int32_t G = p.group;
    const int32_t rows_total = n * G;
    const int32_t row0 = qt * kRowsPerWG;
    if (row0 >= rows_total) return;                // uniform for the work-group

    const int32_t my_row = row0 + wave * 32 + col;
    const bool row_valid = my_row < rows_total;
    const int32_t row_c = row_valid ? my_row : rows_total - 1;
    const int32_t node = row_c / G;
    const int32_t g = row_c - node * G;
    const int32_t head = kvh * G + g;
    const int64_t t = int64_t(node_base) + node;
    const uint64_t *mrow = p.mask + t * p.words_per_row;

    // ---- KV tile range of this split -----------------------------------------------------------------------
    const int ntp = (P + kKeysPerTile - 1) / kKeysPerTile;
    const int ntd = (n + kKeysPerTile - 1) / kKeysPerTile;
    const int nt = ntp + ntd;
    const int per_split = (nt + p.splits - 1) / p.splits;
    const int t_begin = split * per_split;
    const int t_end = min(nt, t_begin + per_split);

    // draft tiles that no row of this work-group can see are skipped: bit j of `live` = tile j has a set bit
    uint64_t live = 0;
    for (int j = 0; j < ntd; ++j) {
        const uint64_t w = row_valid ? mrow[j] : 0;
        if (__syncthreads_or(w != 0)) live |= uint64_t(1) << (j & 63);
    }
    auto tile_live = [&](int ti) -> bool { return ti < ntp || ((live >> ((ti - ntp) & 63)) & 1); };

    // ---- Q fragments: B operand of S^T = K Q^T; lane holds Q[row][ks*16 + 8*half .. +7] ------------------------
    bf16x8 qf[KS];
    {
        const __bf16 *qp = p.q + t * p.q_ts + int64_t(head) * p.q_hs + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }

    floatx16 acc_o[MBD];
#pragma unroll
    for (int i = 0; i < MBD; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc_o[i][j] = 0.f;
    float m_run = kMInit;
    float l_run = 0.f;

    // ---- global -> register staging of one K/V tile ---------------------------------------------------------
    const __bf16 *k_seq = p.k + p.kv_offsets[b] * p.kv_ts + int64_t(kvh) * p.kv_hs;
    const __bf16 *v_seq = p.v + p.kv_offsets[b] * p.kv_ts + int64_t(kvh) * p.kv_hs;
    const int ld_row = tid / CHUNKS;
    const int ld_chunk = tid % CHUNKS;
    const int32_t last_row = P + n - 1;            // last K/V row of the sequence: loads are clamped to it
    u32x4 kreg[K_PASSES], vreg[2 * V_PASSES];
    uint64_t word_next = 0;

    auto tile_first_row = [&](int ti) -> int32_t { return ti < ntp ? ti * kKeysPerTile : P + (ti - ntp) * kKeysPerTile; };
    auto issue_loads = [&](int ti) {
        const int32_t r0 = tile_first_row(ti);
#pragma unroll
        for (int ps = 0; ps < K_PASSES; ++ps) {
            const int32_t r = min(r0 + ps * ROWS_PER_PASS + ld_row, last_row);
            kreg[ps] = *reinterpret_cast<const u32x4 *>(k_seq + int64_t(r) * p.kv_ts + ld_chunk * 8);
        }
#pragma unroll
        for (int ps = 0; ps < V_PASSES; ++ps) {
            const int32_t ra = min(r0 + 2 * (ps * ROWS_PER_PASS + ld_row), last_row);
            const int32_t rb = min(ra + 1, last_row);
            vreg[2 * ps] = *reinterpret_cast<const u32x4 *>(v_seq + int64_t(ra) * p.kv_ts + ld_chunk * 8);
            vreg[2 * ps + 1] = *reinterpret_cast<const u32x4 *>(v_seq + int64_t(rb) * p.kv_ts + ld_chunk * 8);
        }
        if (ti >= ntp) word_next = mrow[ti - ntp];
    };
    auto stage_to_lds = [&]() {
#pragma unroll
        for (int ps = 0; ps < K_PASSES; ++ps) {
            const int r = ps * ROWS_PER_PASS + ld_row;
            *reinterpret_cast<u32x4 *>(lds_k + k_lds_row(r) * L::kKRowBytes + ld_chunk * 16) = kreg[ps];
        }
#pragma unroll
        for (int ps = 0; ps < V_PASSES; ++ps) {
            const int pr = ps * ROWS_PER_PASS + ld_row;
            const u32x4 a = vreg[2 * ps], c = vreg[2 * ps + 1];
            u32x4 lo, hi;   // channel-major pairs: (key 2pr, key 2pr+1) for channels 8*chunk .. +7
            lo[0] = __builtin_amdgcn_perm(c[0], a[0], 0x05040100u);
            lo[1] = __builtin_amdgcn_perm(c[0], a[0], 0x07060302u);
            lo[2] = __builtin_amdgcn_perm(c[1], a[1], 0x05040100u);
            lo[3] = __builtin_amdgcn_perm(c[1], a[1], 0x07060302u);
            hi[0] = __builtin_amdgcn_perm(c[2], a[2], 0x05040100u);
            hi[1] = __builtin_amdgcn_perm(c[2], a[2], 0x07060302u);
            hi[2] = __builtin_amdgcn_perm(c[3], a[3], 0x05040100u);
            hi[3] = __builtin_amdgcn_perm(c[3], a[3], 0x07060302u);
            char *dst = lds_v + pr * L::kVRowBytes + ld_chunk * 32;
            *reinterpret_cast<u32x4 *>(dst) = lo;
            *reinterpret_cast<u32x4 *>(dst + 16) = hi;
        }
    };

    // first live tile of the range
    int ti = t_begin;
    while (ti < t_end && !tile_live(ti)) ++ti;
    if (ti < t_end) issue_loads(ti);

    while (ti < t_end) {
        int tn = ti + 1;
        while (tn < t_end && !tile_live(tn)) ++tn;

        __syncthreads();                 // every wave is done reading the previous tile
        stage_to_lds();
        const uint64_t word = word_next;
        __syncthreads();
        if (tn < t_end) issue_loads(tn); // in flight while this tile is computed

        // ---- S^T = K Q^T : two 32-key blocks x 32 query rows ----------------------------------------------
        floatx16 acc_s[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int j = 0; j < 16; ++j) acc_s[mb][j] = 0.f;
            const char *kp = lds_k + (mb * 32 + col) * L::kKRowBytes + half * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kp + ks * 32);
                acc_s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], acc_s[mb], 0, 0, 0);
            }
        }

        // ---- mask: only draft tiles and the ragged last prefix tile ----------------------------------------
        // accumulator register i of block mb is key  mb*32 + 16*(i/8) + 8*half + i%8  of the tile
        const bool is_draft = ti >= ntp;
        const int32_t valid = is_draft ? min(kKeysPerTile, n - (ti - ntp) * kKeysPerTile)
                                       : min(kKeysPerTile, P - ti * kKeysPerTile);
        if (is_draft || valid < kKeysPerTile) {
            uint64_t vis = is_draft ? word : ~uint64_t(0);
            if (valid < kKeysPerTile) vis &= (uint64_t(1) << valid) - 1;
            vis >>= 8 * half;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = mb * 32 + 16 * (i / 8) + (i % 8);
                    if (!((vis >> key) & 1)) acc_s[mb][i] = -__builtin_inff();
                }
        }

        // ---- online softmax (per-lane row; the other 16 keys of each block live in lane^32) -----------------
        float mx = acc_s[0][0];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc_s[mb][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        if (__any(m_new > m_run)) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2e);
            l_run *= alpha;
#pragma unroll
            for (int i = 0; i < MBD; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc_o[i][j] *= alpha;
            m_run = m_new;
        }
        const float neg_m = -m_run * p.scale_log2e;
        bf16x8 pf[4];
        float psum = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float e = __builtin_amdgcn_exp2f(fmaf(acc_s[mb][i], p.scale_log2e, neg_m));
                psum += e;
                pf[mb * 2 + i / 8][i % 8] = (__bf16)e;
            }
        l_run += psum;

        // ---- O^T += V^T P^T ---------------------------------------------------------------------------------
#pragma unroll
        for (int ks2 = 0; ks2 < 4; ++ks2) {
            const char *vp = lds_v + (ks2 * 8 + 4 * half) * L::kVRowBytes + col * 4;
#pragma unroll
            for (int mbd = 0; mbd < MBD; ++mbd) {
                u32x4 raw;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    raw[jj] = *reinterpret_cast<const uint32_t *>(vp + jj * L::kVRowBytes + mbd * 128);
                const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
                acc_o[mbd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[ks2], acc_o[mbd], 0, 0, 0);
            }
        }
        ti = tn;
    }

    // ---- epilogue ------------------------------------------------------------------------------------------
    // accumulator register i of channel block mbd is channel  mbd*32 + 8*(i/4) + 4*half + i%4
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (!row_valid) return;
    if (p.splits == 1) {
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        __bf16 *op = p.o + t * p.o_ts + int64_t(head) * p.o_hs + 4 * half;
#pragma unroll
        for (int mbd = 0; mbd < MBD; ++mbd)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(acc_o[mbd][i4 * 4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + mbd * 32 + i4 * 8) = x;
            }
        if (p.lse && half == 0)
            p.lse[t * p.num_q_heads + head] =
                l_tot > 0.f ? m_run * p.scale + __logf(l_tot) : -__builtin_inff();
    } else {
        const int64_t prow = (int64_t(split) * p.total_nodes + t) * p.num_q_heads + head;
        float *op = p.part_o + prow * D + 4 * half;
#pragma unroll
        for (int mbd = 0; mbd < MBD; ++mbd)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                floatx4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = acc_o[mbd][i4 * 4 + e];
                *reinterpret_cast<floatx4 *>(op + mbd * 32 + i4 * 8) = x;
            }
        if (half == 0) {
            floatx2 ml;
            ml[0] = m_run;
            ml[1] = l_tot;
            *reinterpret_cast<floatx2 *>(p.part_ml + prow * 2) = ml;
        }
    }
}

// Merge of the split partials, one wavefront per (node, head) row, splits taken in index order.
template <int D>
__global__ __launch_bounds__(256) void dag_attention_combine_kernel(const AttnParams p) {
    const int lane = threadIdx.x & 63;
    const int64_t row = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);      // t * Hq + head
    const int64_t rows = int64_t(p.total_nodes) * p.num_q_heads;
    if (row >= rows) return;
    const int64_t t = row / p.num_q_heads;
    const int head = int(row - t * p.num_q_heads);

    float m = kMInit;
    for (int s = 0; s < p.splits; ++s) m = fmaxf(m, p.part_ml[(int64_t(s) * rows + row) * 2]);
    constexpr int PER_LANE = D / 64;
    float acc[PER_LANE];
#pragma unroll
    for (int e = 0; e < PER_LANE; ++e) acc[e] = 0.f;
    float l = 0.f;
    for (int s = 0; s < p.splits; ++s) {
        const int64_t prow = int64_t(s) * rows + row;
        const float ms = p.part_ml[prow * 2], ls = p.part_ml[prow * 2 + 1];
        const float w = __builtin_amdgcn_exp2f((ms - m) * p.scale_log2e);
        l = fmaf(ls, w, l);
#pragma unroll
        for (int e = 0; e < PER_LANE; ++e) acc[e] = fmaf(p.part_o[prow * D + lane * PER_LANE + e], w, acc[e]);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    __bf16 *op = p.o + t * p.o_ts + int64_t(head) * p.o_hs + lane * PER_LANE;
#pragma unroll
    for (int e = 0; e < PER_LANE; ++e) op[e] = (__bf16)(acc[e] * inv);
    if (p.lse && lane == 0) p.lse[row] = l > 0.f ? m * p.scale + __logf(l) : -__builtin_inff();
}

// ---------------------------------------------------------------------------------------------- host side

static int q_tiles_of(const gsd_attn_desc &d) {
    const int group = d.num_q_heads / d.num_kv_heads;
    return (d.max_nodes * group + kRowsPerWG - 1) / kRowsPerWG;
}

int attention_bf16_splits(const gsd_attn_desc &d) {
    const int nt_max = (d.max_prefix + kKeysPerTile - 1) / kKeysPerTile + (d.max_nodes + kKeysPerTile - 1) / kKeysPerTile;
    int splits = d.num_splits;
    if (splits <= 0) {
        // aim for about two work-groups per compute unit; never fewer than 4 KV tiles per split
        const int64_t base = int64_t(q_tiles_of(d)) * d.batch * d.num_kv_heads;
        splits = int((512 + base - 1) / base);
        const int cap = nt_max / 4 > 0 ? nt_max / 4 : 1;
        if (splits > cap) splits = cap;
    }
    if (splits > nt_max) splits = nt_max;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    return splits;
}

size_t attention_bf16_workspace(const gsd_attn_desc &d, int splits) {
    if (splits <= 1) return 0;
    return size_t(splits) * d.total_nodes * d.num_q_heads * (size_t(d.head_dim) + 2) * sizeof(float);
}

hipError_t launch_attention_bf16(const gsd_attn_desc &d, int splits, hipStream_t stream) {
    AttnParams p;
    p.q = (const __bf16 *)d.q; p.o = (__bf16 *)d.o; p.lse = d.lse;
    p.k = (const __bf16 *)d.k; p.v = (const __bf16 *)d.v;
    p.kv_offsets = d.kv_offsets; p.prefix_lens = d.prefix_lens; p.node_offsets = d.node_offsets; p.mask = d.mask;
    p.part_o = (float *)d.workspace;
    p.part_ml = p.part_o ? p.part_o + size_t(splits) * d.total_nodes * d.num_q_heads * d.head_dim : nullptr;
    p.q_ts = d.q_token_stride; p.q_hs = d.q_head_stride; p.o_ts = d.o_token_stride; p.o_hs = d.o_head_stride;
    p.kv_ts = d.kv_token_stride; p.kv_hs = d.kv_head_stride;
    p.batch = d.batch; p.total_nodes = d.total_nodes; p.max_nodes = d.max_nodes; p.num_q_heads = d.num_q_heads;
    p.num_kv_heads = d.num_kv_heads; p.group = d.num_q_heads / d.num_kv_heads; p.words_per_row = d.words_per_row;
    p.q_tiles = q_tiles_of(d);
    p.splits = splits;
    p.total_wg = p.q_tiles * splits * d.batch * d.num_kv_heads;
    p.wg_per_xcd = (p.total_wg + 7) / 8;
    p.scale = d.softmax_scale;
    p.scale_log2e = d.softmax_scale * kLog2e;

    const dim3 grid(p.wg_per_xcd * 8), block(kThreads);
    if (d.head_dim == 128)
        hipLaunchKernelGGL(dag_attention_bf16_kernel<128>, grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL(dag_attention_bf16_kernel<64>, grid, block, 0, stream, p);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (splits > 1) {
        const int64_t rows = int64_t(d.total_nodes) * d.num_q_heads;
        const dim3 cgrid((unsigned)((rows + 3) / 4));
        if (d.head_dim == 128)
            hipLaunchKernelGGL(dag_attention_combine_kernel<128>, cgrid, dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(dag_attention_combine_kernel<64>, cgrid, dim3(256), 0, stream, p);
        err = hipGetLastError();
    }
    return err;
}

}  // namespace gsd
