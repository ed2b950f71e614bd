// bf16 DAG-masked flash attention for gfx950 (paper Sections 4.1 / 5.4: one verifier pass over the flattened
// token graph; every draft node attends to the whole context and to its visible draft nodes).
//
// Shape of the work.  All G = Hq/Hkv query heads of a KV head share its K/V rows and (per node) the same mask
// row, so the (node, head) pairs of one (sequence, KV head) are packed into one row space r = node*G + g and
// cut into tiles of 256 rows (128 when a group has fewer than 256); a work-group of 8 (4) wavefronts owns one tile
// (32 rows per wave) and walks the KV axis in tiles of 64 keys: first the prefix tiles (no mask arithmetic, only the ragged last tile is bounded),
// then the draft tiles, one 64-bit mask word per row per tile; a draft tile whose word is zero for every row
// of the work-group is skipped outright.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  Scores are computed TRANSPOSED,
// S^T = K . Q^T, so that a lane owns one query row (column n = lane%32) and 16 keys per 32-key block: the row sum
// is an in-lane loop plus one exchange between the wave's halves, and a rescale factor is a per-lane scalar for
// the O^T = V^T . P^T accumulators, which have the same column ownership.  The S^T accumulator registers are
// converted to bf16 and fed straight back as the B operand of the second contraction: K rows sit in LDS in the
// order that makes each lane's 8 consecutive accumulator registers 8 consecutive keys.
//
// Softmax.  softmax_scale is applied in fp32 to the raw dot products (one fused multiply-add per score, which also
// subtracts the row's offset).  No running max is kept: the offset is set by the first tile and then only watched
// through the tile sums; see kSumRaise below.  Rows whose scores leave the range that scheme can follow are computed
// again, exactly, at the end of the kernel.
//
// Data movement.  K and V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
// no register staging); both are double-buffered.  Rows keep their 16-byte chunks XOR-swizzled (K by row%16, V
// by 4*(row%4) at head_dim 128) so that the 128-bit K reads and the 64-bit transposing V reads (ds_read_b64_tr_b16, which hands
// each lane four consecutive keys of one channel from a row-major tile) are free of bank conflicts.
//
// Schedule.  The loop is a hand-laid software pipeline: while the matrix pipe computes the scores of tile i+1
// the vector ALU exponentiates the second half of tile i's scores; while the matrix pipe accumulates P.V of tile i
// the vector ALU exponentiates the first half of tile i+1's.  Two barriers per tile, each followed by the prefetch
// of the buffer just freed.
//
// Small problems are split along the KV axis (gsd_attn_desc.num_splits); a split writes unnormalised fp32
// partials (O, running max, running sum) and a second kernel merges them in split order.
#include <mutex>
#include <type_traits>

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

constexpr int kKeysPerTile = 64;     // keys per KV tile = one mask word
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMInit = -1e30f;     // finite stand-in for -inf: the offset stored for a partial without any visible key
// A row's offset is not its running max: it is a guess (the true max of the first tile) that is corrected only when
// a tile's probabilities leave a harmless range.  Per lane, the 32 probabilities of a tile add up to less than
// kSumRaise whenever none of its shifted scores exceeds 9 (log2); a larger sum raises the offset for the tiles that
// follow.  A sum that is not below kSumPoison (a score more than ~64 above the offset, an overflow, a NaN) or a row
// total below kSumTiny (an offset more than ~64 above every score) cannot be trusted in fp32: such a row is flagged
// and computed again by the exact, slow path of the epilogue.
constexpr float kSumRaise = 16384.0f;
constexpr float kSumPoison = 0x1p64f;
constexpr float kSumTiny = 0x1p-64f;

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
    float *part_ml;     // [splits][T][Hq][2]  (offset in the log2 domain, sum of 2^(score - offset))
    int64_t q_ts, q_hs, o_ts, o_hs, kv_ts, kv_hs;
    int32_t batch, total_nodes, max_nodes, num_q_heads, num_kv_heads, group, words_per_row;
    int32_t q_tiles;    // row tiles per (sequence, KV head)
    int32_t splits;
    int32_t wg_per_xcd; // ceil(batch * num_kv_heads / 8) * q_tiles * splits
    float scale_log2e;  // softmax_scale * log2(e)
};

template <int D>
struct Lds {
    static constexpr int kRowBytes = D * 2;                       // one K or V row, unpadded (swizzled instead)
    static constexpr int kTileBytes = kKeysPerTile * kRowBytes;
    static constexpr int kTotal = 4 * kTileBytes;                 // K and V, both double-buffered
};

// position of actual key row r (0..63) inside the LDS K tile: bits 2 and 3 of r swapped (an involution)
__device__ __forceinline__ int k_lds_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// Nothing may be moved across this point by the instruction scheduler: the loop body below is laid out by hand
// as slices of one matrix instruction, one or two LDS reads for a later slice and a few softmax operations, so
// that the matrix pipe and the vector ALU of a wave run side by side.
#define GSD_SLICE_END() __builtin_amdgcn_sched_barrier(0)

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// max over the two 32-lane halves of a wavefront, in every lane
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// One 16-byte-per-lane global -> LDS copy: lane l's 16 bytes at gbase + voff land at LDS byte lds_base + 16*l.
// Issued as inline assembly so that the compiler's wait-count pass does not serialise later LDS reads behind
// it; completion is awaited by hand (dma_wait) before the barrier that publishes the tile.
__device__ __forceinline__ void dma16(const void *gbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                 :: "s"(gbase), "v"(voff), "s"(lds_base) : "memory");
}
// The same with the LDS address as a scalar base plus a constant, added inside: given one scalar per destination
// the compiler keeps them all live across the loop (sixteen at four copies per tile and wave) and spills them.
__device__ __forceinline__ void dma16_at(const void *gbase, uint32_t voff, uint32_t lds_base, int lds_const) {
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                 :: "s"(gbase), "v"(voff), "s"(lds_base), "i"(lds_const) : "memory", "scc");
}
template <int N> __device__ __forceinline__ void dma_wait() {   // at most N vector-memory operations in flight
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// A wave-uniform 64-bit value, forced into scalar registers (the copies above take their base address from there;
// a uniform value loaded through the vector memory path would otherwise stay in vector registers).
__device__ __forceinline__ int64_t uniform64(int64_t x) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(x)));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(x) >> 32));
    return int64_t((uint64_t(hi) << 32) | lo);
}
// Work-group barrier as bare assembly: the compiler's own barrier is preceded by a wait for every outstanding LDS
// read, which would undo the reads issued ahead of it on purpose (their results are awaited where they are used).
__device__ __forceinline__ void wg_barrier() {
    asm volatile("s_barrier" ::: "memory");
}

// Matrix instructions written out for the one-wave-per-SIMD variant.  With 512 registers per lane the compiler
// selects the accumulator-register form for every matrix instruction it emits itself, and then moves every score
// into an ordinary register before the softmax can touch it.  Written out, the score accumulators stay in ordinary
// registers ("v") and only the output accumulators and the query fragments, which the vector ALU never reads in
// the loop, live in accumulator registers ("a").  The compiler does not know these are matrix instructions, so
// the two places where the vector ALU reads their results soon after them wait by hand (mfma_settle).
__device__ __forceinline__ void mfma_v_acc(floatx16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_v_init(floatx16 &acc, const bf16x8 &a, const bf16x8 &b) {   // starts a chain from zero
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_a_acc(floatx16 &acc, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// at least 16 issue cycles: longer than the 12 the vector ALU must keep away from an 8-pass matrix result
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 7\n\ts_nop 7" ::: "memory"); }

// NW wavefronts per work-group, each owning RBW blocks of 32 query rows.
//   <4 waves, 2 blocks>  256 rows, one work-group per CU, one wave per SIMD with the whole register file: every K/V
//                        fragment read from LDS feeds two matrix instructions, so the instructions a wave has to
//                        issue per matrix instruction (LDS reads, waits, copies, loop control) halve.  On this chip a
//                        wave issues about one instruction every four cycles and two waves of a SIMD do not overlap
//                        their matrix and vector work, so that count is what bounds the kernel.
//   <8 waves, 1 block>   256 rows, two waves per SIMD.
//   <4 waves, 1 block>   128 rows, two work-groups per CU: wastes less when a (sequence, KV head) has few rows.
template <int D, int NW, int RBW>
__global__ __launch_bounds__(NW * 64, RBW == 2 ? 1 : 8 / NW) void dag_attention_bf16_kernel(const AttnParams p) {
    constexpr int kThreads = NW * 64;
    constexpr int kRowsPerWG = NW * 32 * RBW;
    constexpr bool ASM_MFMA = RBW == 2;
    constexpr int KS = D / 16;          // k-steps of the first contraction
    constexpr int MBD = D / 32;         // 32-channel blocks of the output
    constexpr int NQK = 2 * KS;         // matrix instructions of S^T = K Q^T per tile
    constexpr int NPV = 4 * MBD;        // matrix instructions of O^T += V^T P^T per tile
    constexpr int CHUNKS = D / 8;       // 16-byte chunks per K/V row
    // Of a lane's 32 scores per tile, the first B_SCORES are converted in phase B, the rest in phase A.  Measured
    // at 4, 8, 12 and 16: within half a percent of each other.
    constexpr int B_SCORES = 16;
    static_assert(B_SCORES % 2 == 0 && B_SCORES >= 2 && B_SCORES <= 16, "");
    using L = Lds<D>;
    constexpr int RB = L::kRowBytes;
    constexpr int RPI = 1024 / RB;      // tile rows moved by one wave-wide 16-byte-per-lane copy
    constexpr int IPW = (L::kTileBytes / 1024) / (kThreads / 64);   // such copies per wave per tile
    // K-row swizzle: a bitwise-linear function of the LDS row position (so it distributes over the sums below)
    auto k_swz = [](int m) __attribute__((always_inline)) -> int { return D == 128 ? (m & 15) : ((m >> 1) & 7); };
    __shared__ __attribute__((aligned(1024))) char lds[L::kTotal];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    // buffer x of K at lds + x*kTileBytes, buffer x of V at lds + (2+x)*kTileBytes

    // ---- which piece of work: XCD-aware decode of the linear work-group id --------------------------------
    // Hardware deals consecutive work-group ids round-robin to the 8 XCDs.  A (sequence, KV head) group stays on
    // one XCD, in consecutive slots, so that its row tiles run together and share the K/V stream in that XCD's L2;
    // the groups themselves are dealt round-robin (group g on XCD g % 8), so that the KV heads of one sequence,
    // which all have that sequence's length, are spread over the XCDs and ragged batches load them evenly.
    const int hw = blockIdx.x;
    const int per_group = p.q_tiles * p.splits;
    const int xcd_slot = hw >> 3;
    const int group_id = (xcd_slot / per_group) * 8 + (hw & 7);      // b * Hkv + kvh
    if (group_id >= p.batch * p.num_kv_heads) return;
    const int within = xcd_slot % per_group;
    const int qt = within % p.q_tiles;
    const int split = within / p.q_tiles;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int b = group_id / p.num_kv_heads;
    const int kvh = group_id - b * p.num_kv_heads;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;        // which 8-wide k group / which 4-row group of the accumulator
    const int col = lane & 31;         // query row inside the wave's 32

    const int32_t node_base = p.node_offsets[b];
    const int32_t n = min(p.node_offsets[b + 1] - node_base, p.max_nodes);   // never trust past the stated bound
    const int32_t P = p.prefix_lens[b];
    const int32_t G = p.group;
    const int32_t rows_total = n * G;
    const int32_t row0 = qt * kRowsPerWG;
    if (row0 >= rows_total) return;                // uniform for the work-group

    // row block rb of this wave: rows row0 + (wave*RBW + rb)*32 .. +31, this lane's row is +col
    auto row_of = [&](int rb) __attribute__((always_inline)) -> int32_t { return row0 + (wave * RBW + rb) * 32 + col; };
    auto row_is_valid = [&](int rb) __attribute__((always_inline)) -> bool { return row_of(rb) < rows_total; };
    auto node_of = [&](int rb) __attribute__((always_inline)) -> int32_t {   // rows past the end stand in for the last row
        return min(row_of(rb), rows_total - 1) / G;
    };
    auto head_of = [&](int rb) __attribute__((always_inline)) -> int32_t {
        const int32_t r = min(row_of(rb), rows_total - 1);
        return kvh * G + (r - (r / G) * G);
    };

    // ---- KV tile range of this split -----------------------------------------------------------------------
    const int ntp = (P + kKeysPerTile - 1) / kKeysPerTile;
    const int ntd = (n + kKeysPerTile - 1) / kKeysPerTile;
    const int nt = ntp + ntd;
    const int per_split = (nt + p.splits - 1) / p.splits;
    const int t_begin = split * per_split;
    const int t_end = min(nt, t_begin + per_split);
    const int full_end = min(t_end, P / kKeysPerTile);      // tiles below this index need no mask at all

    // draft tiles that no row of this work-group can see are skipped: bit j of `live` = tile j has a set bit
    // The rows' mask words are parked in LDS on the way: fetched from global memory inside the loop they would sit
    // behind the tile copies in the in-order memory counter and stall the wave for a full memory round trip.
    constexpr int kMaxWords = GSD_MAX_NODES_PER_SEQ / 64;
    __shared__ uint64_t mask_lds[kRowsPerWG * kMaxWords];
    // words of row block rb: my_mask + rb*32*kMaxWords (both halves of the wave write the same words)
    uint64_t *my_mask = mask_lds + (wave * RBW * 32 + col) * kMaxWords;
    uint64_t live = 0;
    {
        // All words of a row are fetched by unconditional loads (the word index is clamped, the value masked
        // afterwards): guarded loads become a branch and a full wait per word, eight memory round trips in a row.
        uint32_t lane_live = 0;          // bit j: a row of this lane sees a node of draft tile j
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
            const uint64_t *mrow = p.mask + (int64_t(node_base) + node_of(rb)) * p.words_per_row;
            const bool ok = row_is_valid(rb);
            uint64_t words[kMaxWords];
#pragma unroll
            for (int j = 0; j < kMaxWords; ++j) words[j] = mrow[min(j, p.words_per_row - 1)];
#pragma unroll
            for (int j = 0; j < kMaxWords; ++j) {
                const uint64_t w = (ok && j < ntd) ? words[j] : 0;
                my_mask[rb * 32 * kMaxWords + j] = w;
                lane_live |= uint32_t(w != 0) << j;
            }
        }
        // one exchange for the whole work-group: every wave publishes which tiles its rows see
        __shared__ uint32_t wave_live[NW];
        uint32_t mine = 0;
#pragma unroll
        for (int j = 0; j < kMaxWords; ++j)
            if (__ballot((lane_live >> j) & 1u)) mine |= 1u << j;
        if (lane == 0) wave_live[wave] = mine;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) live |= wave_live[w];
    }
    // smallest live tile index > ti inside the split's range, or t_end
    auto next_live = [&](int ti) __attribute__((always_inline)) -> int {
        const int u = ti + 1;
        if (u >= t_end) return t_end;
        if (u < ntp) return u;
        const uint64_t rem = live >> (u - ntp);
        if (rem == 0) return t_end;
        const int v = u + __builtin_ctzll(rem);
        return v < t_end ? v : t_end;
    };

    // ---- Q fragments: B operand of S^T = K Q^T; lane holds Q[row][ks*16 + 8*half .. +7] ------------------------
    bf16x8 qf[RBW][KS];
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        const __bf16 *qp = p.q + (int64_t(node_base) + node_of(rb)) * p.q_ts + int64_t(head_of(rb)) * p.q_hs + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[rb][ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
        // resident in the accumulator file from here on (otherwise each use copies its fragment over again)
        if (ASM_MFMA) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[rb][ks]));
        }
    }

    floatx16 acc_o[RBW][MBD];
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
        for (int i = 0; i < MBD; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc_o[rb][i][j] = 0.f;
    // Softmax state of a row.  The matrix pipe delivers raw dot products; one fused multiply-add per score applies
    // softmax_scale*log2(e) in fp32 and subtracts the row's offset, and the result goes straight into exp2.  Any
    // offset gives the same softmax, so no running max is kept: the offset is set from the first tile and afterwards
    // only the sum of each tile's probabilities is looked at (one compare per tile).  When it has grown large the
    // wave takes a rare branch that touches scalars only: the offset goes up by the sum's exponent for the tiles that
    // follow, the running sum is rescaled, and the factor is parked for the output accumulators, which are multiplied
    // once the tile in flight has been added to them.  What this cannot handle (see kSumPoison, kSumTiny) flags the row.
    float nm[RBW];             // minus the row's offset (log2 domain)
    float l_run[RBW];          // this lane's share of the running sum (the other half lives in lane^32)
    float sum_carry[RBW];      // sum of the held tile's probabilities converted so far (those taken in phase B)
    float alpha_now[RBW];      // factor for the output accumulators, due at the start of the next phase B
    float alpha_next[RBW];     // the same, due one phase B later (the tile whose sum tripped is still to be added)
    bool poison[RBW];          // per lane: this row needs the exact path
    bool pend_now = false, pend_next = false;      // wave-uniform: something other than one is parked there
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        nm[rb] = 0.f;
        l_run[rb] = 0.f;
        sum_carry[rb] = 0.f;
        alpha_now[rb] = 1.f;
        alpha_next[rb] = 1.f;
        poison[rb] = false;
    }
    const float c_log2 = p.scale_log2e;

    // ---- global -> LDS copies of K/V tiles ----------------------------------------------------------------------
    // Copy j of this wave fills LDS rows (wave*IPW + j)*RPI .. +RPI-1 of the tile buffer; lane l lands in row
    // +l/CHUNKS, 16-byte slot l%CHUNKS, and therefore fetches the chunk that the swizzle assigns to that slot.
    static_assert(RPI % 4 == 0 && (RPI == 4 || RPI == 8), "row bookkeeping below assumes 4 or 8 rows per copy");
    static_assert(IPW >= 1 && IPW * (kThreads / 64) * 1024 == L::kTileBytes, "the waves' copies must tile the buffer");
    const int64_t kv_elem_off = uniform64(p.kv_offsets[b] * p.kv_ts + int64_t(kvh) * p.kv_hs);
    const __bf16 *k_seq = p.k + kv_elem_off;
    const __bf16 *v_seq = p.v + kv_elem_off;
    const uint32_t row_stride_bytes = uint32_t(p.kv_ts) * 2u;
    const int32_t last_row = P + n - 1;            // last K/V row of the sequence: loads are clamped to it
    const uint32_t wave_lds = lds_base + wave * IPW * 1024;     // where this wave's first copy of a tile lands in buffer 0
    // Copy j = 0 decides everything: later copies only add compile-time constants (rows) or flip one chunk bit.
    const int32_t m0 = wave * IPW * RPI + lane / CHUNKS;          // LDS row position filled by copy 0
    const int slot = lane % CHUNKS;
    const uint32_t k_src_chunk0 = uint32_t(slot ^ k_swz(m0)) * 16u;
    const uint32_t v_src_chunk = uint32_t((slot ^ ((CHUNKS / 4) * (m0 & 3))) & (CHUNKS - 1)) * 16u;  // RPI % 4 == 0
    auto tile_first_row = [&](int ti) __attribute__((always_inline)) -> int32_t {
        return ti < ntp ? ti * kKeysPerTile : P + (ti - ntp) * kKeysPerTile;
    };
    // copy j (0..IPW-1) of this wave's share of tile ti into K / V buffer `buf`
    auto dma_k_one = [&](int ti, int buf, int j) __attribute__((always_inline)) {
        // source row of LDS position m0 + j*RPI: the row permutation is bitwise, and m0, j*RPI share no bits
        const uint32_t r = uint32_t(min(tile_first_row(ti) + k_lds_row(m0) + k_lds_row(j * RPI), last_row));
        const uint32_t chunk = k_src_chunk0 ^ uint32_t(k_swz(j * RPI) * 16);
        dma16_at(k_seq, __umul24(r, row_stride_bytes) + chunk, wave_lds + buf * L::kTileBytes, j * 1024);
    };
    auto dma_v_one = [&](int ti, int buf, int j) __attribute__((always_inline)) {
        const uint32_t r = uint32_t(min(tile_first_row(ti) + m0 + j * RPI, last_row));
        dma16_at(v_seq, __umul24(r, row_stride_bytes) + v_src_chunk, wave_lds + (2 + buf) * L::kTileBytes, j * 1024);
    };
    // The same copies over a run of consecutive full prefix tiles (all 64 rows exist, no clamp): every lane keeps
    // the byte offset of its next chunk and adds one tile's worth after each copy, which is all the address
    // arithmetic left (the general form costs a chain of about ten dependent scalar instructions per copy).
    uint32_t k_run[IPW], v_run[IPW];
    const uint32_t tile_stride_bytes = uint32_t(kKeysPerTile) * row_stride_bytes;
    auto start_full_run = [&](int k_tile, int v_tile) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) {
            k_run[j] = uint32_t(k_tile * kKeysPerTile + k_lds_row(m0) + k_lds_row(j * RPI)) * row_stride_bytes +
                       (k_src_chunk0 ^ uint32_t(k_swz(j * RPI) * 16));
            v_run[j] = uint32_t(v_tile * kKeysPerTile + m0 + j * RPI) * row_stride_bytes + v_src_chunk;
        }
    };
    auto dma_k_one_full = [&](int buf, int j) __attribute__((always_inline)) {
        dma16_at(k_seq, k_run[j], wave_lds + buf * L::kTileBytes, j * 1024);
        k_run[j] += tile_stride_bytes;
    };
    auto dma_v_one_full = [&](int buf, int j) __attribute__((always_inline)) {
        dma16_at(v_seq, v_run[j], wave_lds + (2 + buf) * L::kTileBytes, j * 1024);
        v_run[j] += tile_stride_bytes;
    };
    auto dma_k = [&](int ti, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) dma_k_one(ti, buf, j);
    };
    auto dma_v = [&](int ti, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < IPW; ++j) dma_v_one(ti, buf, j);
    };

    // ---- LDS read addresses -------------------------------------------------------------------------------------
    // The LDS has 64 four-byte banks: a 128-bit read is served 16 lanes at a time, a 64-bit read 32 lanes at a
    // time, and the lanes served together must not meet in a bank.  Hence the swizzles: a K row at LDS position
    // m keeps logical 16-byte chunk c in slot c ^ k_swz(m) (16 consecutive rows fill the 16 slots of a 256-byte
    // bank line exactly once); a V row r keeps chunk c in slot c ^ (CHUNKS/4)*(r % 4).
    //
    // K fragment (ks, mb): 16 bytes = channels ks*16 + 8*half .. +7 of LDS row mb*32 + col, i.e. logical chunk
    // ks*2 + half.  Its byte address is (row base + (half ^ k_swz(col))*16) ^ (ks*32): one per-lane value per ks.
    uint32_t k_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        k_off[ks] = uint32_t(col * RB + ((half ^ k_swz(col)) * 16)) ^ uint32_t(ks * 32);
    // V fragment (ks2, mbd), part h2: transposing 8-byte read.  Within a 16-lane group, lane s supplies the
    // address of row kv0 + s/4, channels d0 + 4*(s%4) .. +3, and receives keys kv0 .. kv0+3 of channel d0 + s;
    // d0 = mbd*32 + 16*(group&1), kv0 = ks2*16 + 8*(group>>1) + 4*h2, so row % 4 = s/4.  Logical chunk
    // mbd*4 + y with y = 2*(group&1) + (s%4)/2; its address is (per-lane value) ^ (mbd*64).
    uint32_t v_off[MBD];
    {
        const int sl = lane & 15, grp = lane >> 4;
        const int y = (grp & 1) * 2 + (sl & 3) / 2;
        const uint32_t v0 = uint32_t((8 * (grp >> 1) + sl / 4) * RB + (((y ^ ((CHUNKS / 4) * (sl / 4))) & (CHUNKS - 1)) * 16) +
                                     (sl & 1) * 8);
#pragma unroll
        for (int x = 0; x < MBD; ++x) v_off[x] = v0 ^ uint32_t(x * 64);
    }
    auto k_frag = [&](int buf, int idx) __attribute__((always_inline)) -> bf16x8 {
        const int mb = idx & 1, ks = idx >> 1;
        const char *ptr = lds + buf * L::kTileBytes + mb * 32 * RB + k_off[ks];
        return *reinterpret_cast<const bf16x8 *>(ptr);
    };
    auto v_frag = [&](int buf, int idx) __attribute__((always_inline)) -> bf16x8 {
        const int ks2 = idx / MBD, mbd = idx % MBD;
        const char *ptr = lds + (2 + buf) * L::kTileBytes + ks2 * 16 * RB + v_off[mbd];
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4 *)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)ptr);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4 *)(uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)(ptr + 4 * RB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // mask of tile `ti` applied to the raw scores: register i of block mb is key mb*32 + 16*(i/8) + 8*half + i%8
    auto apply_mask = [&](floatx16 (&sc)[2], int ti, int rb) __attribute__((always_inline)) {
        const bool is_draft = ti >= ntp;
        const int32_t valid = is_draft ? min(kKeysPerTile, n - (ti - ntp) * kKeysPerTile)
                                       : min(kKeysPerTile, P - ti * kKeysPerTile);
        uint64_t vis = is_draft ? my_mask[rb * 32 * kMaxWords + ti - ntp] : ~uint64_t(0);
        if (valid < kKeysPerTile) vis &= (uint64_t(1) << valid) - 1;
        vis >>= 8 * half;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = mb * 32 + 16 * (i / 8) + (i % 8);
                if (!((vis >> key) & 1)) sc[mb][i] = -__builtin_inff();
            }
    };
    // The first tile sets the offset: the max of its raw (masked) scores, in the exponent's units.  A row that sees
    // no key of this tile keeps the guess 0.
    auto first_offset = [&](floatx16 (&sc)[2], int rb) __attribute__((always_inline)) {
        float mx0 = -__builtin_inff(), mx1 = -__builtin_inff();
#pragma unroll
        for (int e = 0; e < 32; e += 4) {
            mx0 = max3(mx0, sc[e / 16][e % 16], sc[(e + 1) / 16][(e + 1) % 16]);
            mx1 = max3(mx1, sc[(e + 2) / 16][(e + 2) % 16], sc[(e + 3) / 16][(e + 3) % 16]);
        }
        const float mx = max_across_halves(fmaxf(mx0, mx1));
        nm[rb] = mx > -__builtin_inff() ? -(mx * c_log2) : 0.f;
    };
    // The rare branch after a tile whose sum `tot` tripped in some lane of the wave.  Per row (both halves of the
    // wave agree on everything decided here): a sum that cannot be trusted flags the row; otherwise a large sum
    // raises the offset by its exponent, for the tiles that follow.  Adds the tile's sum to the running sum.
    auto adjust = [&](float tot, int rb) __attribute__((always_inline)) {
        const bool bad_here = !(tot < kSumPoison);
        const auto sw = __builtin_amdgcn_permlane32_swap(uint32_t(bad_here), uint32_t(bad_here), false, false);
        poison[rb] = poison[rb] | ((sw[0] | sw[1]) != 0);
        const float big = max_across_halves(bad_here ? 0.f : tot);
        const float delta = big < kSumRaise ? 0.f : float(__builtin_amdgcn_frexp_expf(big));   // big < 2^delta
        const float alpha = __builtin_amdgcn_exp2f(-delta);                                    // exact, 1 if nothing moves
        nm[rb] -= delta;
        l_run[rb] = (l_run[rb] + (bad_here ? 0.f : tot)) * alpha;
        alpha_next[rb] = alpha;
    };

    // ---- the software pipeline ---------------------------------------------------------------------------------
    // Live tiles are taken in order i = 0, 1, ...; at the top of step i
    //   registers   raw (masked) scores of tile i, the first B_SCORES of each lane already converted with the row's
    //               offset, and the first four K fragments of tile i+1
    //   LDS         K(i+1) in K buffer (i+1)&1 and V(i) in V buffer i&1, complete and published
    //   in flight   the copy of K(i+2) -> K buffer i&1 (V(i+1) is issued during phase A)
    // Step i:  phase A: scores of tile i+1 on the matrix pipe while the vector ALU turns the scores of tile i
    //                   into bf16 probabilities; its last slices read the first V fragments of tile i; then the
    //                   check of the tile's sum and, rarely, the repair
    //          wait for K(i+2)'s copy, barrier (now the K buffer just read may be refilled with K(i+3), in phase B)
    //          phase B: O^T += V^T P^T on the matrix pipe while the vector ALU converts the first scores of tile
    //                   i+1 (masked first if that tile needs it); its last slices read the first K fragments of
    //                   tile i+2
    //          wait for V(i+1)'s copy, barrier (now the V buffer just read may be refilled, in the next phase A)
    // Each wait leaves the youngest copy in flight (IPW operations); near the end of the range, where that copy does
    // not exist, it waits for everything.  A tile is thus published one barrier before the phase that consumes it,
    // which is what lets that phase's first fragments be read ahead of the barrier in front of it.
    u32x4 pf[RBW][4];          // bf16 probabilities of the tile, two per register, in accumulator-register order
    // The first four fragments of a phase are read from LDS during the last slices of the phase before it, ahead
    // of the barrier between them (the tile they come from was published one barrier earlier), so that the matrix
    // pipe does not idle for an LDS round trip after every barrier.
    bf16x8 kpre[4], vpre[4];

    // matrix instruction idx (0..NQK-1) of a tile's scores for row block rb: the first of each chain starts from zero
    auto score_mfma = [&](floatx16 &acc, const bf16x8 &kfrag, int rb, int idx) __attribute__((always_inline)) {
        if (ASM_MFMA) {
            if (idx < 2) mfma_v_init(acc, kfrag, qf[rb][idx >> 1]);
            else mfma_v_acc(acc, kfrag, qf[rb][idx >> 1]);
        } else {
            floatx16 zero;
#pragma unroll
            for (int j = 0; j < 16; ++j) zero[j] = 0.f;
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag, qf[rb][idx >> 1], idx < 2 ? zero : acc, 0, 0, 0);
        }
    };
    // raw scores e and e+1 of `sc` -> bf16 probabilities 2^(score*scale*log2(e) - offset), stored in accumulator-
    // register order, and added to the lane's sum.  Plain v_add_f32 on purpose: measured on this chip, ordinary vector
    // instructions (add, fma, max3, cvt_pk_bf16) issue in the shadow of a running matrix instruction for free and
    // v_exp_f32 for three quarters, but v_dot2c_f32_bf16 (one instruction per pair) runs on the matrix pipe itself,
    // takes ~2.5x as long as an add and overlaps with nothing.
    auto convert_pair_with = [&](floatx16 (&sc)[2], int e, float &sum, int rb, float minus_offset) __attribute__((always_inline)) {
        floatx2 x;
        x[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e / 16][e % 16], c_log2, minus_offset));
        x[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[(e + 1) / 16][(e + 1) % 16], c_log2, minus_offset));
        const bf16x2 pr = __builtin_convertvector(x, bf16x2);
        pf[rb][e / 8][(e / 2) % 4] = __builtin_bit_cast(uint32_t, pr);
        sum += x[0] + x[1];
        asm volatile("" : "+v"(sum));      // keeps the two additions in this slice (they would be collected behind the last one)
    };
    auto convert_pair = [&](floatx16 (&sc)[2], int e, float &sum, int rb) __attribute__((always_inline)) {
        convert_pair_with(sc, e, sum, rb, nm[rb]);
    };
    // The same one score at a time, for the loop: the vector work is dealt out evenly, one score behind every matrix
    // instruction (an even score waits in x_hold for its odd neighbour, with which it is packed).
    float x_hold[RBW];
    // Split in two so that nothing waits for an exponential: score e is started (multiply-add, exp2) in one slice
    // and retired (added to the sum, packed with its neighbour) in the slice that starts score e+1.
    float x_new[RBW];
    auto start_one = [&](floatx16 (&sc)[2], int e, int rb) __attribute__((always_inline)) {
        x_new[rb] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e / 16][e % 16], c_log2, nm[rb]));
    };
    auto retire_one = [&](int e, float &sum, int rb) __attribute__((always_inline)) {
        const float x = x_new[rb];
        sum += x;
        asm volatile("" : "+v"(sum));
        if (e & 1) {
            floatx2 xx;
            xx[0] = x_hold[rb];
            xx[1] = x;
            pf[rb][e / 8][(e / 2) % 4] = __builtin_bit_cast(uint32_t, __builtin_convertvector(xx, bf16x2));
        } else {
            x_hold[rb] = x;
        }
    };
    // The exponentials are the vector ALU's heaviest load, so they are split between the two phases: phase B of
    // step i-1 converts scores 0..B_SCORES-1 of tile i (right after it has found the tile's max), phase A of step i
    // converts the rest.  A slice is one K or V fragment's worth of matrix instructions (one per row block).
    //
    // phase A.  HAS_NEXT: also compute the raw scores of the next tile from K buffer `kbuf` into s_next, and spread
    // the copy of the next tile's V (tile `v_tile` into V buffer `v_buf`) over the slices: issued back to back after
    // a barrier, the copies of all the waves queue up in the texture path.  v_cur: V buffer of the current tile.
    auto phase_a = [&](auto has_next_tag, auto full_tag, int kbuf, floatx16 (&sc)[RBW][2], floatx16 (&s_next)[RBW][2], int v_tile, int v_buf, int v_cur) __attribute__((always_inline)) {
        constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;     // the tile being copied is a full prefix tile
        float sum[RBW];
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) sum[rb] = 0.f;
        bf16x8 kf[NQK];
        if (HAS_NEXT) {
#pragma unroll
            for (int x = 0; x < 4; ++x) kf[x] = kpre[x];
        } else {
#pragma unroll
            for (int x = 0; x < 4; ++x) vpre[x] = v_frag(v_cur, x);
        }
        GSD_SLICE_END();
#pragma unroll
        for (int idx = 0; idx < NQK; ++idx) {
            // One sub-slice per row block: its matrix instruction, then the vector work of that row block.  A wave
            // that issues two matrix instructions back to back sits blocked on the second until the pipe is free;
            // with its share of the vector work in between it arrives there about when the pipe does.
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
                if (HAS_NEXT) {
                    score_mfma(s_next[rb][idx & 1], kf[idx], rb, idx);
                    if (rb == RBW - 1) {
                        if (idx + 4 < NQK) kf[idx + 4] = k_frag(kbuf, idx + 4);
                        else vpre[idx + 4 - NQK] = v_frag(v_cur, idx + 4 - NQK);   // phase B's first reads, ahead of the barrier
                        if (idx % (NQK / IPW) == 1) {
                            if (FULL) dma_v_one_full(v_buf, idx / (NQK / IPW));
                            else dma_v_one(v_tile, v_buf, idx / (NQK / IPW));
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 32 - B_SCORES; ++u)            // score B_SCORES + u goes into slice u*NQK/(32-B_SCORES)
                    if ((u * NQK) / (32 - B_SCORES) == idx) {
                        if (u > 0) retire_one(B_SCORES + u - 1, sum[rb], rb);
                        start_one(sc[rb], B_SCORES + u, rb);
                    }
                GSD_SLICE_END();
            }
        }
        // keep the conversions in this phase: without a use here the compiler sinks them next to their first use in
        // phase B, behind the barrier, and the overlap with the matrix pipe is lost
        float tot[RBW];
        bool trip = false;
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) retire_one(31, sum[rb], rb);
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
            asm volatile("" : "+v"(pf[rb][1]), "+v"(pf[rb][2]), "+v"(pf[rb][3]), "+v"(sum[rb]));
            if (HAS_NEXT) asm volatile("" : "+v"(s_next[rb][0]), "+v"(s_next[rb][1]));
            tot[rb] = sum_carry[rb] + sum[rb];
            trip |= !(tot[rb] < kSumRaise);         // also true for a sum that is not a number
        }
        if (__builtin_expect(__any(trip), 0)) {     // rare, wave-uniform, scalars only
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) adjust(tot[rb], rb);
            pend_next = true;
        } else {
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) l_run[rb] += tot[rb];
        }
    };

    // phase B.  vbuf: V buffer of the current tile.  HAS_NEXT: meanwhile the vector ALU masks s_next if `next_tile`
    // is not a full prefix tile and converts its scores 0..B_SCORES-1 (from the slice at which pf[0], then pf[1], have
    // been consumed), leaving their sum in sum_carry.
    // COPY_K spreads the copy of tile `k_tile` into K buffer `k_buf` over the slices.
    auto phase_b = [&](auto has_next_tag, auto copy_k_tag, auto full_tag, int vbuf, floatx16 (&s_next)[RBW][2], int next_tile, int k_tile, int k_buf, bool k_ahead, int k_next_buf) __attribute__((always_inline)) {
        constexpr bool COPY_K = decltype(copy_k_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
        constexpr int CONV_FIRST = MBD;                 // first slice that converts: pf[.][0] is last read by slice MBD-1
        // pf[.][1] (scores 8..15) is last read by slice 2*MBD-1 and is first rewritten when score 9 has been converted
        static_assert(B_SCORES <= 8 || CONV_FIRST + (9 * (NPV - CONV_FIRST)) / B_SCORES >= 2 * MBD,
                      "probabilities of the current tile would be overwritten before they are used");
        if (__builtin_expect(pend_now | pend_next, 0)) {    // an offset moved one or two tiles ago
            if (pend_now) {
                if (ASM_MFMA) mfma_settle();
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb) {
#pragma unroll
                    for (int x = 0; x < MBD; ++x) {
                        // take the value from the accumulator file and hand the product back to it inside the branch,
                        // or the copies out of and into that file are hoisted in front of the branch and run every step
                        if (ASM_MFMA) asm volatile("" : "+a"(acc_o[rb][x]));
#pragma unroll
                        for (int j = 0; j < 16; ++j) acc_o[rb][x][j] *= alpha_now[rb];
                        if (ASM_MFMA) asm volatile("" : "+a"(acc_o[rb][x]));
                    }
                }
                if (ASM_MFMA) mfma_settle();
            }
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
                alpha_now[rb] = alpha_next[rb];
                alpha_next[rb] = 1.f;
            }
            pend_now = pend_next;
            pend_next = false;
        }
        bf16x8 vf[NPV];
#pragma unroll
        for (int x = 0; x < 4; ++x) vf[x] = vpre[x];
        if (ASM_MFMA && HAS_NEXT) mfma_settle();            // the scores written by phase A's last matrix instructions
        if (HAS_NEXT && !FULL && next_tile >= full_end) {   // FULL: the next tile is a full prefix tile too
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) apply_mask(s_next[rb], next_tile, rb);
        }
        float sum[RBW];
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) sum[rb] = 0.f;
        GSD_SLICE_END();
#pragma unroll
        for (int idx = 0; idx < NPV; ++idx) {
            const int ks2 = idx / MBD, mbd = idx % MBD;
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {      // sub-slices as in phase A
                if (ASM_MFMA) mfma_a_acc(acc_o[rb][mbd], vf[idx], __builtin_bit_cast(bf16x8, pf[rb][ks2]));
                else acc_o[rb][mbd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[idx], __builtin_bit_cast(bf16x8, pf[rb][ks2]), acc_o[rb][mbd], 0, 0, 0);
                if (rb == RBW - 1) {
                    if (idx + 4 < NPV) vf[idx + 4] = v_frag(vbuf, idx + 4);
                    else if (HAS_NEXT && k_ahead) kpre[idx + 4 - NPV] = k_frag(k_next_buf, idx + 4 - NPV);   // next phase A's first reads
                    if (COPY_K && idx % (NPV / IPW) == 1) {
                        if (FULL) dma_k_one_full(k_buf, idx / (NPV / IPW));
                        else dma_k_one(k_tile, k_buf, idx / (NPV / IPW));
                    }
                }
                if (HAS_NEXT) {
#pragma unroll
                    for (int u = 0; u < B_SCORES; ++u)             // score u goes into slice CONV_FIRST + u*(NPV-CONV_FIRST)/B_SCORES
                        if (CONV_FIRST + (u * (NPV - CONV_FIRST)) / B_SCORES == idx) {
                            if (u > 0) retire_one(u - 1, sum[rb], rb);
                            start_one(s_next[rb], u, rb);
                        }
                }
                GSD_SLICE_END();
            }
        }
        if (HAS_NEXT) {
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) retire_one(B_SCORES - 1, sum[rb], rb);
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
                asm volatile("" : "+v"(pf[rb][0]), "+v"(pf[rb][1]), "+v"(sum[rb]));
                sum_carry[rb] = sum[rb];
            }
        }
    };

    using True = std::integral_constant<bool, true>;
    using False = std::integral_constant<bool, false>;

    int c0 = next_live(t_begin - 1);
    if (c0 < t_end) {
        int c1 = next_live(c0), c2 = next_live(c1), c3 = next_live(c2);
        floatx16 sa[RBW][2], sb[RBW][2];
        // prologue: K(0), V(0), K(1) on their way; scores and max of tile 0; then V(1), K(2)
        dma_k(c0, 0);
        dma_v(c0, 0);
        if (c1 < t_end) {
            dma_k(c1, 1);
            dma_wait<2 * IPW>();
        } else {
            dma_wait<0>();
        }
        wg_barrier();
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
#pragma unroll
            for (int idx = 0; idx < NQK; ++idx)
                score_mfma(sa[rb][idx & 1], k_frag(0, idx), rb, idx);
            if (ASM_MFMA) mfma_settle();
            if (c0 >= full_end) apply_mask(sa[rb], c0, rb);
            first_offset(sa[rb], rb);
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < B_SCORES; e += 2) convert_pair(sa[rb], e, sum, rb);
            sum_carry[rb] = sum;
        }
        wg_barrier();          // K buffer 0 has been read by every wave
        if (c2 < t_end) {
            dma_k(c2, 0);
            dma_wait<IPW>();   // V(0) and K(1) have landed
        } else {
            dma_wait<0>();
        }
        wg_barrier();
        if (c1 < t_end) {
#pragma unroll
            for (int x = 0; x < 4; ++x) kpre[x] = k_frag(1, x);
        }

        int i = 0;
        // one step with the current scores in `cur`, leaving the next tile's scores in `nxt`.  STEADY: tiles
        // i+2 and i+3 exist, so nothing in the step is conditional and two copies stay in flight at each wait.
        // FAST: all tiles up to i+4 are full prefix tiles: no search for the next live tile, no clamp in the copies.
        auto step = [&](auto steady_tag, auto fast_tag, floatx16 (&cur)[RBW][2], floatx16 (&nxt)[RBW][2]) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_tag)::value;
            constexpr bool FAST = decltype(fast_tag)::value;
            phase_a(True{}, fast_tag, (i + 1) & 1, cur, nxt, c1, (i + 1) & 1, i & 1);   // also starts the copy of V(i+1)
            if (STEADY) dma_wait<IPW>(); else dma_wait<0>();             // K(i+2) has landed (V(i) did a barrier ago)
            wg_barrier();
            if (!STEADY && c3 < t_end) dma_k(c3, (i + 1) & 1);
            phase_b(True{}, steady_tag, fast_tag, i & 1, nxt, c1, c3, (i + 1) & 1, STEADY || c2 < t_end, i & 1);   // steady: also copies K(i+3)
            if (STEADY) dma_wait<IPW>(); else dma_wait<0>();             // V(i+1) has landed
            wg_barrier();
            c0 = c1; c1 = c2; c2 = c3; c3 = FAST ? c3 + 1 : next_live(c3);
            ++i;
        };
        // steady state over the prefix, two steps per trip so that the two score buffers swap roles without copies
        if (c3 + 2 < full_end) start_full_run(c3, c1);
        while (c3 + 2 < full_end) {
            step(True{}, True{}, sa, sb);
            step(True{}, True{}, sb, sa);
        }
        while (c3 < t_end) {       // the rest of the steady state: the next live tile has to be searched for
            step(True{}, False{}, sa, sb);
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) sa[rb][mb] = sb[rb][mb];
        }
        while (c1 < t_end) {       // the last steps: no more tiles to prefetch
            step(False{}, False{}, sa, sb);
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) sa[rb][mb] = sb[rb][mb];
        }
        // last tile: nothing left to prefetch or to score
        phase_a(False{}, False{}, 0, sa, sb, 0, 0, i & 1);
        phase_b(False{}, False{}, False{}, i & 1, sb, 0, 0, 0, false, 0);
    }

    // ---- epilogue ------------------------------------------------------------------------------------------
    // accumulator register i of channel block mbd is channel  mbd*32 + 8*(i/4) + 4*half + i%4
    if (ASM_MFMA) mfma_settle();
    uint32_t redo[RBW];        // wave-uniform: bit r = row r of row block rb goes through the exact path
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32, 64);
        // A row total that is tiny (or zero, or not a number) although the row sees a key of this KV range means the
        // offset sat far above every score: what was flushed to zero on the way may have mattered.
        bool flagged = poison[rb];
        if (!(l_tot >= kSumTiny)) {
            bool sees = t_begin < min(t_end, ntp);
#pragma unroll
            for (int j = 0; j < kMaxWords; ++j)
                sees |= j + ntp >= t_begin && j + ntp < t_end && my_mask[rb * 32 * kMaxWords + j] != 0;
            flagged |= sees;
        }
        const bool valid = row_is_valid(rb);
        const uint64_t votes = __ballot(flagged && valid);
        redo[rb] = uint32_t(votes) | uint32_t(votes >> 32);
        if (!valid || flagged) continue;
        const int64_t t = int64_t(node_base) + node_of(rb);
        const int32_t head = head_of(rb);
        // a factor may still be parked for the accumulators (the last tile's sum tripped, or the one before it)
        const float parked = alpha_now[rb] * alpha_next[rb];
        if (p.splits == 1) {
            const float inv = l_tot > 0.f ? parked / l_tot : 0.f;
            __bf16 *op = p.o + t * p.o_ts + int64_t(head) * p.o_hs + 4 * half;
#pragma unroll
            for (int mbd = 0; mbd < MBD; ++mbd)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    bf16x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (__bf16)(acc_o[rb][mbd][i4 * 4 + e] * inv);
                    *reinterpret_cast<bf16x4 *>(op + mbd * 32 + i4 * 8) = x;
                }
            if (p.lse && half == 0)
                p.lse[t * p.num_q_heads + head] =
                    l_tot > 0.f ? (-nm[rb] + __log2f(l_tot)) * 0.6931471805599453f : -__builtin_inff();
        } else {
            const int64_t prow = (int64_t(split) * p.total_nodes + t) * p.num_q_heads + head;
            float *op = p.part_o + prow * D + 4 * half;
#pragma unroll
            for (int mbd = 0; mbd < MBD; ++mbd)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    floatx4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = acc_o[rb][mbd][i4 * 4 + e] * parked;
                    *reinterpret_cast<floatx4 *>(op + mbd * 32 + i4 * 8) = x;
                }
            if (half == 0) {
                floatx2 ml;
                ml[0] = l_tot > 0.f ? -nm[rb] : kMInit;
                ml[1] = l_tot;
                *reinterpret_cast<floatx2 *>(p.part_ml + prow * 2) = ml;
            }
        }
    }

    // ---- exact path for flagged rows (rare; correctness, not speed) ---------------------------------------------
    // One row at a time, the whole wave on it: scores of up to kExactKeys keys at once, one key per lane, fp32 dot
    // products against the query row parked in LDS; then one channel pair per lane walks those keys with a true
    // running max.  Uses the K/V tile buffers, which every wave has finished with after the barrier.
    bool any_redo = false;
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) any_redo |= redo[rb] != 0;
    wg_barrier();
    if (__builtin_expect(!any_redo, 1)) return;
    constexpr int kExactKeys = 512;
    constexpr int PER = D / 64;                    // output channels per lane
    static_assert(L::kTotal / NW >= int((D + kExactKeys) * sizeof(float)), "per-wave share of the tile buffers");
    float *q_lds = reinterpret_cast<float *>(lds + wave * (L::kTotal / NW));
    float *s_lds = q_lds + D;
    const int32_t pk0 = min(P, t_begin * kKeysPerTile), pk1 = min(P, t_end * kKeysPerTile);
    const int32_t dn0 = min(n, max(t_begin - ntp, 0) * kKeysPerTile), dn1 = min(n, max(t_end - ntp, 0) * kKeysPerTile);
    const int32_t n_prefix = pk1 - pk0, n_keys = n_prefix + (dn1 - dn0);
#pragma unroll
    for (int rb = 0; rb < RBW; ++rb) {
        for (uint32_t todo = redo[rb]; todo != 0; todo &= todo - 1) {
            const int r = __builtin_ctz(todo);
            const int32_t row = row0 + (wave * RBW + rb) * 32 + r;
            const int32_t node = row / G, head = kvh * G + (row - node * G);
            const int64_t t = int64_t(node_base) + node;
            const uint64_t *mw = mask_lds + (wave * RBW * 32 + rb * 32 + r) * kMaxWords;
            const __bf16 *qp = p.q + t * p.q_ts + int64_t(head) * p.q_hs;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the row before has been read out of LDS
            for (int d = lane; d < D; d += 64) q_lds[d] = (float)qp[d];
            float m = -__builtin_inff(), l = 0.f, o[PER];
#pragma unroll
            for (int e = 0; e < PER; ++e) o[e] = 0.f;
            // key x of the range: prefix position pk0 + x, then draft node dn0 + (x - n_prefix)
            auto kv_row = [&](int32_t x) -> int32_t { return x < n_prefix ? pk0 + x : P + dn0 + (x - n_prefix); };
            auto visible = [&](int32_t x) -> bool {
                if (x < n_prefix) return true;
                const int32_t nd = dn0 + (x - n_prefix);
                return (mw[nd >> 6] >> (nd & 63)) & 1;
            };
            for (int32_t base = 0; base < n_keys; base += kExactKeys) {
                const int32_t cnt = min(kExactKeys, n_keys - base);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // q_lds written, s_lds of the chunk before read
                float cmax = -__builtin_inff();
                for (int32_t j = lane; j < cnt; j += 64) {
                    float sc = -__builtin_inff();
                    if (visible(base + j)) {
                        const __bf16 *kp = k_seq + int64_t(kv_row(base + j)) * p.kv_ts;
                        float dot = 0.f;
                        for (int d = 0; d < D; d += 8) {
                            const bf16x8 kk = *reinterpret_cast<const bf16x8 *>(kp + d);
#pragma unroll
                            for (int z = 0; z < 8; ++z) dot = __builtin_fmaf((float)kk[z], q_lds[d + z], dot);
                        }
                        sc = dot * c_log2;
                    }
                    s_lds[j] = sc;
                    cmax = fmaxf(cmax, sc);
                }
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off, 64));
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the chunk's scores are in LDS
                if (!(cmax > -__builtin_inff())) continue;          // nothing visible in this chunk
                const float m_new = fmaxf(m, cmax);
                const float shrink = m > -__builtin_inff() ? __builtin_amdgcn_exp2f(m - m_new) : 0.f;
                m = m_new;
                l *= shrink;
#pragma unroll
                for (int e = 0; e < PER; ++e) o[e] *= shrink;
                for (int32_t j = 0; j < cnt; ++j) {
                    const float sc = s_lds[j];                      // the same address in every lane
                    if (!(sc > -__builtin_inff())) continue;
                    const float pj = __builtin_amdgcn_exp2f(sc - m);
                    l += pj;
                    const __bf16 *vp = v_seq + int64_t(kv_row(base + j)) * p.kv_ts + lane * PER;
#pragma unroll
                    for (int e = 0; e < PER; ++e) o[e] = __builtin_fmaf(pj, (float)vp[e], o[e]);
                }
            }
            if (p.splits == 1) {
                const float inv = l > 0.f ? 1.f / l : 0.f;
                __bf16 *op = p.o + t * p.o_ts + int64_t(head) * p.o_hs + lane * PER;
#pragma unroll
                for (int e = 0; e < PER; ++e) op[e] = (__bf16)(o[e] * inv);
                if (p.lse && lane == 0)
                    p.lse[t * p.num_q_heads + head] =
                        l > 0.f ? (m + __log2f(l)) * 0.6931471805599453f : -__builtin_inff();
            } else {
                const int64_t prow = (int64_t(split) * p.total_nodes + t) * p.num_q_heads + head;
#pragma unroll
                for (int e = 0; e < PER; ++e) p.part_o[prow * D + lane * PER + e] = o[e];
                if (lane == 0) {
                    p.part_ml[prow * 2] = l > 0.f ? m : kMInit;
                    p.part_ml[prow * 2 + 1] = l;
                }
            }
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
        const float w = __builtin_amdgcn_exp2f(ms - m);
        l = fmaf(ls, w, l);
#pragma unroll
        for (int e = 0; e < PER_LANE; ++e) acc[e] = fmaf(p.part_o[prow * D + lane * PER_LANE + e], w, acc[e]);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    __bf16 *op = p.o + t * p.o_ts + int64_t(head) * p.o_hs + lane * PER_LANE;
#pragma unroll
    for (int e = 0; e < PER_LANE; ++e) op[e] = (__bf16)(acc[e] * inv);
    if (p.lse && lane == 0) p.lse[row] = l > 0.f ? (m + __log2f(l)) * 0.6931471805599453f : -__builtin_inff();
}

// ---------------------------------------------------------------------------------------------- host side

// Shape of a work-group: (wavefronts, 32-row blocks per wavefront).  256-row tiles (8 waves x 1 block) when a
// (sequence, KV head) can fill them, else 128-row tiles (4 x 1).  gsd_attn_desc.wg_waves overrides: 4 -> 4 x 1,
// 8 -> 8 x 1, 64 -> 4 x 2 (measured slower: with one wave per SIMD nothing fills a wave's issue stalls).
struct WgShape { int waves, blocks; };
static WgShape shape_of(const gsd_attn_desc &d) {
    if (d.wg_waves == 4) return {4, 1};
    if (d.wg_waves == 8) return {8, 1};
    if (d.wg_waves == 64) return {4, 2};
    const int group = d.num_q_heads / d.num_kv_heads;
    return d.max_nodes * group >= 256 ? WgShape{8, 1} : WgShape{4, 1};
}

static int q_tiles_of(const gsd_attn_desc &d) {
    const int group = d.num_q_heads / d.num_kv_heads;
    const WgShape sh = shape_of(d);
    const int rows_per_wg = sh.waves * sh.blocks * 32;
    return (d.max_nodes * group + rows_per_wg - 1) / rows_per_wg;
}

int attention_bf16_splits(const gsd_attn_desc &d) {
    const int nt_max = (d.max_prefix + kKeysPerTile - 1) / kKeysPerTile + (d.max_nodes + kKeysPerTile - 1) / kKeysPerTile;
    int splits = d.num_splits;
    if (splits <= 0) {
        // The split count that a small timing model likes best (microseconds, fitted to this kernel on the 256-CU
        // part: ~10 per work-group outside its tile loop, 1.0 per tile of a 4-wave work-group and 1.65 of an 8-wave
        // one at head_dim 128, work-groups beyond what the chip holds at once run in further rounds; the partials
        // and the merge kernel cost 2 + S + rows/1024 * (0.9 + 0.13 S)).  Splitting only pays when few work-groups
        // would otherwise walk a long KV axis; never fewer than 4 KV tiles per split.
        const WgShape sh = shape_of(d);
        const double wgs = double(q_tiles_of(d)) * d.batch * d.num_kv_heads;
        const double resident = 256.0 * (sh.waves == 8 || sh.blocks == 2 ? 1 : 2);
        const double t_tile = (sh.waves == 8 ? 1.65 : sh.blocks == 2 ? 2.4 : 1.0) * d.head_dim / 128.0;
        const double rows_k = double(d.total_nodes) * d.num_q_heads / 1024.0;
        const int cap = nt_max / 4 > 0 ? (nt_max / 4 < 64 ? nt_max / 4 : 64) : 1;
        double best = 0;
        for (int s = 1; s <= cap; ++s) {
            const double rounds = double(int64_t((wgs * s + resident - 1) / resident));
            const double t = rounds * (10.0 + double((nt_max + s - 1) / s) * t_tile) +
                             (s > 1 ? 2.0 + s + rows_k * (0.9 + 0.13 * s) : 0.0);
            if (s == 1 || t < best) {
                best = t;
                splits = s;
            }
        }
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

// Scratch of the allocation-free entry point (gsd_dag_attention_static): the split-KV partials live in this array
// instead of a caller workspace.  Every GPU the library runs on holds its own copy at its own address until the
// process ends.  In host code the array's name is only a handle for the runtime: the device address is asked for
// once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[GSD_STATIC_SCRATCH_BYTES];

hipError_t attention_static_scratch(void **ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *address[kMaxDevices];           // zero-initialised: not asked yet
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if (!address[dev]) {
        void *found = nullptr;
        err = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!found) return hipErrorInvalidSymbol;
        address[dev] = found;
    }
    *ptr = address[dev];
    return hipSuccess;
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
    p.wg_per_xcd = (d.batch * d.num_kv_heads + 7) / 8 * p.q_tiles * splits;
    p.scale_log2e = d.softmax_scale * kLog2e;

    const WgShape sh = shape_of(d);
    const dim3 grid(p.wg_per_xcd * 8), block(sh.waves * 64);
    if (d.head_dim == 128) {
        if (sh.blocks == 2) hipLaunchKernelGGL((dag_attention_bf16_kernel<128, 4, 2>), grid, block, 0, stream, p);
        else if (sh.waves == 8) hipLaunchKernelGGL((dag_attention_bf16_kernel<128, 8, 1>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((dag_attention_bf16_kernel<128, 4, 1>), grid, block, 0, stream, p);
    } else {
        if (sh.blocks == 2) hipLaunchKernelGGL((dag_attention_bf16_kernel<64, 4, 2>), grid, block, 0, stream, p);
        else if (sh.waves == 8) hipLaunchKernelGGL((dag_attention_bf16_kernel<64, 8, 1>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((dag_attention_bf16_kernel<64, 4, 1>), grid, block, 0, stream, p);
    }
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
