// Tree-masked attention of the tree tokens against [KV prefix | tree keys].
//
// bf16 path (MFMA).  Query rows of one kv head are the (node, group head) pairs, packed as
// the N dimension of S^T = K Q^T so that every lane owns ONE query column of the 32x32
// score block: the softmax statistics are lane-local plus one exchange with lane^32.  The
// probabilities come out of the S^T accumulator in exactly the register layout the B
// operand of O^T = V^T P^T wants, so P never leaves registers.  K tiles are staged in LDS
// row-major, V tiles transposed ([d][key], key order permuted to match the accumulator
// layout).  The prefix may be split across workgroups (partial max / sum / O, merged by a
// second kernel) when a batch offers too few (sequence, kv head, row tile) items to fill
// the chip.  The ancestor bitset is applied only to key blocks that contain tree keys.
//
// fp32 path: plain ALU kernel, one wave per (node, head); a correctness path for small
// problems and for head sizes the MFMA path does not cover.

#include "common.hpp"
#include "kernels.hpp"

namespace dt {


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// Global-address-space views: pointers fetched from memory (the per-sequence prefix pointers)
// would otherwise be generic, and generic loads also count against the LDS wait counter.
typedef const __bf16 __attribute__((address_space(1))) *gbf16p;
typedef const bf16x8 __attribute__((address_space(1))) *gbf16x8p;
__device__ __forceinline__ bf16x8 gload8(gbf16p p) { return *(gbf16x8p)p; }
typedef const char __attribute__((address_space(1))) *gbytep;

// LDS transpose read of gfx950 (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane p
// supplies the address of 4 consecutive 16-bit values; with X the concatenation of the 16
// quadruples in lane order, lane i receives X[i], X[16+i], X[32+i], X[48+i].  Pointing lane
// p = 4j+q at row j, columns 4q..4q+3 of a row-major tile therefore hands lane i the column
// i of rows 0..3: a 4x16 -> 16x4 transpose, which is what a K-contiguous MFMA operand needs
// from a matrix stored with the other index contiguous.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4 lds_read_tr4(const __bf16 *p) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)p);
    return __builtin_bit_cast(bf16x4, v);
}

// The same two LDS reads as bare instructions, for loops that keep the wait counters by hand: the
// compiler neither counts them nor guards them with a wait for outstanding global_load_lds traffic
// (it cannot tell a read of one tile from a read of the tile still being filled).  lds_wait<N> lets at
// most N later LDS operations stay outstanding and ties the wait to the register it releases.
__device__ __forceinline__ bf16x8 lds_load128(u32 addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}
// One global_load_lds_dwordx4 with the address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane byte offset, the LDS destination (wave-uniform, the lanes' 16 bytes follow each other) in M0: no
// vector arithmetic per load, and no 64-bit per-lane pointers to keep and advance.
__device__ __forceinline__ void load_to_lds16(const void __attribute__((address_space(1))) *base, u32 lane_off, u32 lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
// a 64-bit value that is the same in every lane, moved to scalar registers where the compiler has not seen that
__device__ __forceinline__ int64_t uniform_i64(int64_t v) {
    const u32 lo = __builtin_amdgcn_readfirstlane((u32)v), hi = __builtin_amdgcn_readfirstlane((u32)((u64)v >> 32));
    return (int64_t)(((u64)hi << 32) | lo);
}
__device__ __forceinline__ gbytep uniform_ptr(gbytep p) { return (gbytep)uniform_i64((int64_t)(uintptr_t)p); }
template <int OFF>
__device__ __forceinline__ bf16x8 lds_load128_at(u32 addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void lds_wait2(bf16x4 &lo, bf16x4 &hi) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(lo), "+v"(hi) : "n"(N));
}
template <int OFF>
__device__ __forceinline__ bf16x4 lds_load_tr4(u32 addr) {
    bf16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8 &v) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(v) : "n"(N));
}

// acc *= alpha, element by element, on an accumulator that stays in the accumulator register file.
// Written out as instructions because any ordinary vector-ALU use of the accumulators inside the
// block loop makes the compiler keep a second copy of all of them in vector registers and move the
// 64 values across in every iteration, although this multiply runs in the first block or two only.
// The idle cycles in front and behind keep the distances the hardware asks for between an MFMA that
// writes or reads an accumulator register and a vector instruction that reads or writes it (the
// compiler does not look inside the instruction group); on this rarely taken path they cost nothing.
__device__ __forceinline__ void acc_scale(f32x16 &acc, float alpha) {
    float t;
#define ACC_SCALE4(i0)                                                                                          \
    {                                                                                                           \
        float e0 = acc[i0], e1 = acc[i0 + 1], e2 = acc[i0 + 2], e3 = acc[i0 + 3];                               \
        asm volatile("s_nop 7\n\ts_nop 7\n\t"                                                                  \
                     "v_accvgpr_read_b32 %4, %0\n\tv_mul_f32 %4, %4, %5\n\tv_accvgpr_write_b32 %0, %4\n\t"     \
                     "v_accvgpr_read_b32 %4, %1\n\tv_mul_f32 %4, %4, %5\n\tv_accvgpr_write_b32 %1, %4\n\t"     \
                     "v_accvgpr_read_b32 %4, %2\n\tv_mul_f32 %4, %4, %5\n\tv_accvgpr_write_b32 %2, %4\n\t"     \
                     "v_accvgpr_read_b32 %4, %3\n\tv_mul_f32 %4, %4, %5\n\tv_accvgpr_write_b32 %3, %4\n\t"     \
                     "s_nop 7"                                                                                  \
                     : "+a"(e0), "+a"(e1), "+a"(e2), "+a"(e3), "=&v"(t)                                         \
                     : "v"(alpha));                                                                             \
        acc[i0] = e0; acc[i0 + 1] = e1; acc[i0 + 2] = e2; acc[i0 + 3] = e3;                                     \
    }
    ACC_SCALE4(0) ACC_SCALE4(4) ACC_SCALE4(8) ACC_SCALE4(12)
#undef ACC_SCALE4
}

// The value of the partner lane (lane ^ 32) next to the own one, without a trip through the LDS
// crossbar: v_permlane32_swap exchanges the upper half of one register with the lower half of another,
// so from two copies of x every lane ends up holding {x[lane], x[lane ^ 32]} in the two registers (in
// either order; layout checked on the device).  Written as an instruction: the compiler's builtin
// returned the same element for both results when they met in one expression.  The waits around it
// cover the vector-write -> swap-read distance the hardware asks for.
__device__ __forceinline__ void half_swap(float x, float &a, float &b) {
    a = x;
    b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float half_swap_max(float x) {
    float a, b;
    half_swap(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float half_swap_sum(float x) {
    float a, b;
    half_swap(x, a, b);
    return a + b;
}

#define ATT_KB 32           // keys per block
#define ATT_ROWS_PER_WAVE 32
#define ATT_WAVES 4
#define ATT_MTILE (ATT_ROWS_PER_WAVE * ATT_WAVES)
#define K_PITCH (128 + 8)   // bf16 elements per K row in LDS (272 B: conflict-free 16 B reads)
// bf16 elements per row of a row-major V tile (288 B): the transposing read takes 4 rows x 32 B
// per 16 lanes, and a pitch of 8 banks modulo 32 spreads those four rows over all 32 banks
#define V_PITCH (128 + 32)
#define VT_PITCH 40         // bf16 elements per V^T row in LDS (80 B)
#define ATT_MAX_SPLITS 16
#define LAZY_LOG2 8.0f        // how far (in powers of two) a probability may exceed 1 before the reference maximum moves

// position of key kk (0..31) inside a V^T row: 16-byte unit (step, lane half) then index,
// mirroring which accumulator registers of S^T a lane holds (rows 8*(i/4) + 4*half + i%4).
__device__ __forceinline__ int vt_pos(int kk) {
    const int step = kk >> 4, q = kk & 15;
    const int half = (q >> 2) & 1, idx = ((q >> 3) << 2) | (q & 3);
    return step * 16 + half * 8 + idx;
}


// 32-bit visibility window of one query over keys t0 .. t0+31, where off = t0 - L (uniform): the
// prefix keys (negative positions) are visible, tree key j is visible iff bit j of the node's
// ancestor set is set (bits at and past the node count are 0, which also hides the padding
// keys past the end of the sequence).
__device__ __forceinline__ u32 vis_window(int off, u64 mask0, u64 mask1) {
    if (off <= -32) return ~0u;
    if (off < 0) return ((u32)mask0 << (-off)) | ((1u << (-off)) - 1u);
    if (off >= 128) return 0u;
    const u64 lo = off < 64 ? mask0 : mask1, hi = off < 64 ? mask1 : 0ull;
    const int sh = off & 63;
    return (u32)((lo >> sh) | (sh ? hi << (64 - sh) : 0ull));
}

// ------------------------------------------------------------------- large-batch kernel -----
// One workgroup = 128 query rows of one (sequence, kv head) (wave w: rows 32w .. 32w+31) times
// one contiguous range of 64-key blocks.  The four waves share each K/V block through LDS, so a
// block crosses the L2 -> LDS path once per 128 rows.  The blocks are loaded straight into LDS
// (global_load_lds_dwordx4: a wave's 64 x 16 B land contiguously, lane after lane), double
// buffered with one barrier per block: the loads of block i+1 are in flight while block i is
// multiplied, and cost neither registers nor LDS-write instructions.
//
// Both tiles are row-major with unpadded 256-byte rows; bank conflicts are avoided by storing
// the 16-byte chunk c of row r at chunk position c ^ f(r) (the permutation is applied on the
// global side: lane p of a row fetches chunk p ^ f(r)):
//   K: f(r) = r % 16.  The A-operand read of S^T = K Q^T has 16 lanes read the same chunk of 16
//      consecutive rows, which now sit at 16 different chunk positions (all 64 banks).
//   V: f(r) = 4 (r % 4) + (r / 4) % 4.  The transposing read takes 4 rows x 64 B per 32 lanes;
//      the four rows now sit in four different 64-byte groups.
#define TILE_KEYS 64
#define TILE_BYTES (TILE_KEYS * 256)     // one K or V tile
#define STAGE_BYTES (2 * TILE_BYTES)     // K tile + V tile of one stage
#define TILE_LDS_BYTES (2 * STAGE_BYTES)
typedef char __attribute__((address_space(3))) *ldsp;

// Where a (sequence, row tile, key range) result goes: the output rows directly when the range is
// the whole sequence, else 128 partial rows (unnormalised O, running max, sum) for the combine.
struct TileDest {
    bool direct;
    float *o;     // [128, D]
    float2 *ml;   // [128]
};

// Rows m0 .. m0+127 of (sequence b, kv head h) against key blocks kb0 .. kb1-1 of that sequence.
// Called by all 256 threads of the workgroup; ends behind a barrier, so calls can follow each other.
template <int D>
__device__ __forceinline__ void tile_segment(const AttnArgs &a, unsigned char *s_dyn, int h, int b, int m0, int kb0,
                                             int kb1, TileDest dst) {
    static_assert(D == 128, "head dim");
    constexpr int KSTEPS = D / 16, DBLK = D / 32;
    const int G = a.Hq / a.Hkv;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int M = N * G;
    const int L = max(a.prefix_len[b], 0);
    const int Tk = L + N;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    const bool active = m0 + 32 * w < M;  // waves past the last row only help with the loads
    const int mq = m0 + 32 * w + col;
    const bool qvalid = mq < M;
    const int node = qvalid ? mq / G : 0;
    const int hq = h * G + (qvalid ? mq % G : 0);

    bf16x8 qreg[KSTEPS];
    {
        const __bf16 *qp = (const __bf16 *)a.q + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) qreg[s] = *(const bf16x8 *)(qp + 16 * s + 8 * half);  // rows past M read node 0: unused
    }
    const u64 mask0 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS];
    const u64 mask1 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS + 1];

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale * 1.4426950408889634f;

    const gbf16p kpre = (gbf16p)a.k_prefix[b] + (int64_t)h * a.kv_stride_head;
    const gbf16p vpre = (gbf16p)a.v_prefix[b] + (int64_t)h * a.kv_stride_head;
    const gbf16p ktree = (gbf16p)a.k_tree + ((int64_t)b * a.TT_cap * a.Hkv + h) * D;
    const gbf16p vtree = (gbf16p)a.v_tree + ((int64_t)b * a.TT_cap * a.Hkv + h) * D;
    const int64_t stok = a.kv_stride_tok, stree = (int64_t)a.Hkv * D;
    // Loading role of a thread, the same for K and V: load i takes key 16 i + tid/16 of the block
    // and lands at chunk position tid%16 of that row, so it fetches chunk (tid%16) ^ f(row); the
    // 16 lanes of a row still cover its 256 bytes.  f(row) does not depend on i (16 | 16 i).
    const int krow = tid >> 4, cpos = tid & 15;
    const int kchunk = cpos ^ krow, vchunk = cpos ^ (((krow & 3) << 2) | (krow >> 2));
    // inside the prefix: a lane's byte offset from the first of its load's sixteen rows (the same for all four loads)
    const u32 koffp = (u32)(krow * stok + 8 * kchunk) * 2u, voffp = (u32)(krow * stok + 8 * vchunk) * 2u;
    const bool small_stride = (int64_t)TILE_KEYS * stok * 2 < ((int64_t)1 << 31);

    // Every load is unconditional.  Keys past the end are read from the last valid row; their
    // scores are masked to -inf below, so their probabilities are exactly 0 and the duplicated V
    // rows contribute nothing.  LDS destination of wave w, load i: rows 16 i + 4 w .. + 3.
    auto fetch = [&](int kb, int stage) {
        const ldsp kdst = (ldsp)s_dyn + stage * STAGE_BYTES + 4 * w * 256;
        const ldsp vdst = kdst + TILE_BYTES;
        if (small_stride && kb * TILE_KEYS + TILE_KEYS <= L) {  // block inside the prefix (uniform test)
            const u32 kl = (u32)(uintptr_t)kdst, vl = (u32)(uintptr_t)vdst;
            const gbytep kbase = uniform_ptr((gbytep)(kpre + (int64_t)kb * TILE_KEYS * stok));
            const gbytep vbase = uniform_ptr((gbytep)(vpre + (int64_t)kb * TILE_KEYS * stok));
            const int64_t step = uniform_i64(16 * stok * 2);  // bytes between the first rows of two loads
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                load_to_lds16(kbase + i * step, koffp, kl + i * 16 * 256);
                load_to_lds16(vbase + i * step, voffp, vl + i * 16 * 256);
            }
        } else {                                                 // block touching the tree keys or the end
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = min(kb * TILE_KEYS + 16 * i + krow, Tk - 1);
                const int64_t o = t < L ? (int64_t)t * stok : (int64_t)(t - L) * stree;
                __builtin_amdgcn_global_load_lds((gbytep)((t < L ? kpre : ktree) + o + 8 * kchunk), kdst + i * 16 * 256,
                                                 16, 0, 0);
                __builtin_amdgcn_global_load_lds((gbytep)((t < L ? vpre : vtree) + o + 8 * vchunk), vdst + i * 16 * 256,
                                                 16, 0, 0);
            }
        }
    };

    // Operand read offsets (bytes inside a tile).
    // K, A operand of S^T: lane (col, half), k-step s reads chunk 2s + half of row 32 j + col.
    u32 koff[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) koff[s] = (u32)(col * 256 + (((2 * s + half) ^ (col & 15)) << 4));
    // V, A operand of O^T = V^T P^T through the transposing read.  Lane (column d = 32 db + col,
    // half) needs, for e = 0..7, V[key 16 st + 8 (e/4) + 4 half + e%4][d]: two reads of 4 keys.  In
    // a 16-lane group lane p16 = 4 r0 + q points at key r0 of the quadruple, columns 4q .. 4q+3 of
    // the group's 16 columns: chunk 4 db + 2 a + q/2 (a = second 16-lane group of the half), byte
    // 8 (q%2) inside it.  Row 16 st + 8 hi + 4 half + r0 has f = 4 r0 + 2 hi + half.
    const int p16 = lane & 15, r0 = p16 >> 2, q4 = p16 & 3, grp = (lane >> 4) & 1;
    u32 voff[DBLK][2];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
            voff[db][hi] = (u32)((8 * hi + 4 * half + r0) * 256 +
                                 (((4 * db + 2 * grp + (q4 >> 1)) ^ (4 * r0 + 2 * hi + half)) << 4) + 8 * (q4 & 1));

    fetch(kb0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's part of the block is in LDS
    __syncthreads();
    for (int kb = kb0; kb < kb1; ++kb) {
        const int cur = (kb - kb0) & 1;
        if (kb + 1 < kb1) fetch(kb + 1, cur ^ 1);  // the other stage was last read before the previous barrier
        if (active) {
            const unsigned char *kt = s_dyn + cur * STAGE_BYTES;  // K tile of this stage, its V tile behind it
            // ---- S^T: 64 keys x 32 queries as two 32x32 blocks -----------------------------------
            // The LDS reads are bare instructions with hand-kept waits: eight K reads (four k-steps of both
            // 32-key halves) stay in flight ahead of the MFMAs, and the first half of the V reads is issued
            // as soon as the K operands are consumed, so that it lands during the softmax.  (Scheduled by the
            // compiler, a read was waited for in full a dozen times per block, and a wait for the next
            // block's global loads stood in front of the first V read.)
            const u32 kl = (u32)(uintptr_t)(ldsp)kt, vl = kl + TILE_BYTES;
            f32x16 sacc[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[j][i] = 0.f;
            bf16x8 ka[16];  // read i: k-step i / 2, half i % 2
#define K_READ(i) ka[i] = lds_load128_at<((i) & 1) * 32 * 256>(kl + koff[(i) >> 1]);
#define QK_STEP(i)                                                                                            \
            lds_wait<((i) < 8 ? 7 : 15 - (i))>(ka[i]);                                                        \
            sacc[(i) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i], qreg[(i) >> 1], sacc[(i) & 1], 0, 0, 0);
            K_READ(0) K_READ(1) K_READ(2) K_READ(3) K_READ(4) K_READ(5) K_READ(6) K_READ(7)
            QK_STEP(0) K_READ(8) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(1) K_READ(9) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(2) K_READ(10) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(3) K_READ(11) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(4) K_READ(12) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(5) K_READ(13) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(6) K_READ(14) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(7) K_READ(15) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(8) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(9) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(10) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(11) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(12) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(13) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(14) __builtin_amdgcn_sched_barrier(0);
            QK_STEP(15) __builtin_amdgcn_sched_barrier(0);
#undef K_READ
#undef QK_STEP
            // V operands of the first 32 keys (MFMA n = 4 st + db of that half): two transposing reads each
            bf16x4 vlo[16], vhi[16];
#define V_READ(n)                                                                                              \
            vlo[n] = lds_load_tr4<(32 * ((n) >> 3) + 16 * (((n) >> 2) & 1)) * 256>(vl + voff[(n) & 3][0]);     \
            vhi[n] = lds_load_tr4<(32 * ((n) >> 3) + 16 * (((n) >> 2) & 1)) * 256>(vl + voff[(n) & 3][1]);
            V_READ(0) V_READ(1) V_READ(2) V_READ(3) V_READ(4) V_READ(5) V_READ(6) V_READ(7)
            __builtin_amdgcn_sched_barrier(0);
            const int tbase = kb * TILE_KEYS;
            if (tbase + TILE_KEYS > L) {  // only blocks that contain tree keys (or the end) need the mask
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const u32 vis = vis_window(tbase + 32 * j - L, mask0, mask1) >> (4 * half);
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        sacc[j][i] = ((vis >> (8 * (i >> 2) + (i & 3))) & 1u) ? sacc[j][i] : -INFINITY;
                }
            }
            // ---- online softmax over the 64 keys (this lane: one query, 32 of the keys) ----------
            float mloc = sacc[0][0];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) mloc = fmaxf(mloc, sacc[j][i]);
            mloc = half_swap_max(mloc);
            // m_run is a reference, not the exact running maximum: it moves only when a block's maximum
            // lies more than LAZY_LOG2 binary orders above it.  Until then probabilities may reach
            // 2^LAZY_LOG2 instead of 1 (harmless in fp32 sums and in bf16's relative precision) and the 64
            // multiplies that rescale the output accumulators are not spent: with unit-variance keys the
            // reference settles on the first block.  (-inf - -inf is NaN: a fully hidden block moves nothing.)
            const bool move = (mloc - m_run) * c > LAZY_LOG2;
            const float m_new = move ? mloc : m_run;
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_use) * c) : 1.0f;  // m_run = -inf -> 0
            const float nmc = -m_use * c;
            float psum = 0.f;
            bf16x8 pb[2][2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[j][i], c, nmc));
                    psum += p;
                    pb[j][i >> 3][i & 7] = (__bf16)p;
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some query of this wave
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
            }
            // ---- O^T += V^T P^T ------------------------------------------------------------------
            // MFMA n (half n / 8, k-step (n / 4) % 2, output block n % 4); the reads of the second half are
            // issued one MFMA at a time behind the first half's MFMAs
#define PV_STEP(n, W)                                                                                          \
            lds_wait2<W>(vlo[n], vhi[n]);                                                                      \
            oacc[(n) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                           \
                __builtin_shufflevector(vlo[n], vhi[n], 0, 1, 2, 3, 4, 5, 6, 7), pb[(n) >> 3][((n) >> 2) & 1], \
                oacc[(n) & 3], 0, 0, 0);
            PV_STEP(0, 0) V_READ(8) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(1, 2) V_READ(9) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(2, 4) V_READ(10) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(3, 6) V_READ(11) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(4, 8) V_READ(12) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(5, 10) V_READ(13) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(6, 12) V_READ(14) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(7, 14) V_READ(15) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(8, 14) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(9, 12) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(10, 10) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(11, 8) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(12, 6) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(13, 4) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(14, 2) __builtin_amdgcn_sched_barrier(0);
            PV_STEP(15, 0)
            // the "memory" clobber keeps the next iteration's loads into this stage behind this block's reads
            asm volatile("" ::: "memory");
#undef PV_STEP
#undef V_READ
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's part of the next block has landed
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------------
    const float l_tot = half_swap_sum(l_run);
    if (!qvalid) return;
    if (dst.direct) {
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        __bf16 *op = (__bf16 *)a.out + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][q * 4 + e] * inv);
                *(bf16x4 *)(op + 32 * db + 8 * q + 4 * half) = o4;
            }
    } else {
        const int rit = 32 * w + col;  // row inside the tile
        float *op = dst.o + (int64_t)rit * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4 o4 = make_float4(oacc[db][q * 4], oacc[db][q * 4 + 1], oacc[db][q * 4 + 2], oacc[db][q * 4 + 3]);
                *(float4 *)(op + 32 * db + 8 * q + 4 * half) = o4;
            }
        if (half == 0) dst.ml[rit] = make_float2(m_run, l_tot);
    }
}

// One workgroup per (kv head, row tile, sequence), the whole key range: enough of them to fill
// the chip several times over.  blockIdx.x = kv head: workgroups are dealt to the 8 XCDs
// round-robin by linear id, so all row tiles of one kv head land on one XCD and share its L2
// copy of that head's K/V.
template <int D>
__global__ __launch_bounds__(256, 2) void attn_tile_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    const int b = blockIdx.z, h = blockIdx.x, m0 = blockIdx.y * ATT_MTILE;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    if (m0 >= N * (a.Hq / a.Hkv)) return;
    const int nb = (max(a.prefix_len[b], 0) + N + TILE_KEYS - 1) / TILE_KEYS;
    TileDest dst;
    dst.direct = true;
    dst.o = nullptr;
    dst.ml = nullptr;
    tile_segment<D>(a, s_dyn, h, b, m0, 0, nb, dst);
}

// ---- balanced schedule for batches that cannot fill the chip with whole (sequence, tile) items --
// Each kv head gets P workgroup slots (two per compute unit over all heads).  Sequences are
// grouped into classes by their number of row tiles m; the key blocks of a class's sequences,
// concatenated in batch order, form its C_m "columns" of cost m each.  Class m is given g_m
// "gangs" of m slots (one per row tile, neighbours in launch order, so the tiles of a sequence walk
// its K/V together and share it in L2); gang j takes columns [j T_m, (j+1) T_m) of the class, with
// T_m = ceil(C_m / g_m), and the g_m are the ones that minimise max_m T_m under sum m g_m <= P.
// A slot therefore works through a few (sequence, tile, key range) segments of near-equal total
// length.  A sequence cut by a range boundary leaves partials: per slot one "head" (its first
// segment, when that sequence began in an earlier gang) and one "tail" (a sequence that began
// here and runs on).  Every wave derives the plan by itself from n_nodes / prefix_len with wave
// operations (sequence b in lane b: batch <= 64; class m in lane m), so no barrier is involved.
struct GangPartial {
    float *o;     // [Hkv, P, 2, 128, D]
    float2 *ml;   // [Hkv, P, 2, 128]
    int *seq;     // [batch, 8]: where sequence b's partials are (written by the attention kernel)
};
enum { GS_FIRST = 0, GS_LAST, GS_BASE, GS_CLS, GS_T, GS_START, GS_WORDS = 8 };

__device__ __forceinline__ int wave_excl_scan_i32(int v, int lane) {
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(x, o, 64);
        if (lane >= o) x += t;
    }
    return x - v;
}

struct GangPlan {
    int mt, nb;        // lane b: row tiles and key blocks of sequence b (0 past the batch)
    int C, g, T;       // lane m: columns, gangs and columns per gang of class m
};

__device__ __forceinline__ GangPlan gang_plan(const AttnArgs &a, int P, int mt_max, int lane) {
    GangPlan p;
    p.mt = 0;
    p.nb = 0;
    if (lane < a.batch) {
        const int N = min(max(a.n_nodes[lane], 1), a.TT_cap);
        p.mt = (N * (a.Hq / a.Hkv) + ATT_MTILE - 1) / ATT_MTILE;
        p.nb = (max(a.prefix_len[lane], 0) + N + TILE_KEYS - 1) / TILE_KEYS;
    }
    p.C = 0;
    for (int m = 1; m <= mt_max; ++m) {
        const int c = wave_sum_i32(p.mt == m ? p.nb : 0);
        if (lane == m) p.C = c;
    }
    const int W = wave_sum_i32(lane * p.C);
    // smallest T with sum_m m ceil(C_m / T) <= P: lane i probes T0 + i.  T = max C_m always fits
    // (the host checks P >= 1 + 2 + .. + mt_max), so the loop ends.
    int T0 = max(1, (W + P - 1) / P), T;
    for (;;) {
        const int t = T0 + lane;
        int slots = 0;
        for (int m = 1; m <= mt_max; ++m) slots += m * ((__builtin_amdgcn_readlane(p.C, m) + t - 1) / t);
        const u64 ok = __ballot(slots <= P);
        if (ok) {
            T = T0 + (int)__builtin_ctzll(ok);
            break;
        }
        T0 += 64;
    }
    p.g = (p.C + T - 1) / T;
    p.T = p.g > 0 ? (p.C + p.g - 1) / p.g : 0;
    return p;
}

template <int D>
__global__ __launch_bounds__(256, 2) void attn_gang_kernel(AttnArgs a, int P, int mt_max, GangPartial part) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    const int h = blockIdx.x, y = blockIdx.y, lane = threadIdx.x & 63;
    const GangPlan p = gang_plan(a, P, mt_max, lane);
    // class, gang and row tile of slot y
    int base = 0, cls = 0;
    for (int m = 1; m <= mt_max; ++m) {
        const int span = m * __builtin_amdgcn_readlane(p.g, m);
        if (cls == 0) {
            if (y < base + span) cls = m;
            else base += span;
        }
    }
    // Slots y, y+P, .. of head 0 also leave sequence y's entry of the table the combine kernel reads:
    // first and last gang of the sequence, first slot, tile count and gang width of its class, and
    // its first column.
    if (h == 0 && threadIdx.x < 64) {
        for (int b = y; b < a.batch; b += P) {
            const int mb = __builtin_amdgcn_readlane(p.mt, b), nbb = __builtin_amdgcn_readlane(p.nb, b);
            int bs = 0;
            for (int m = 1; m < mb; ++m) bs += m * __builtin_amdgcn_readlane(p.g, m);
            const int Tb = __builtin_amdgcn_readlane(p.T, mb);
            const int csb = __builtin_amdgcn_readlane(wave_excl_scan_i32(p.mt == mb ? p.nb : 0, lane), b);
            if (lane == 0) {
                int *e = part.seq + b * GS_WORDS;
                e[GS_FIRST] = csb / Tb;
                e[GS_LAST] = (csb + nbb - 1) / Tb;
                e[GS_BASE] = bs;
                e[GS_CLS] = mb;
                e[GS_T] = Tb;
                e[GS_START] = csb;
            }
        }
    }
    if (cls == 0) return;  // spare slot
    const int j = (y - base) / cls, tile = (y - base) % cls;
    const int Tc = __builtin_amdgcn_readlane(p.T, cls), Cc = __builtin_amdgcn_readlane(p.C, cls);
    const int lo = j * Tc, hi = min(Cc, lo + Tc);
    // first column of every sequence of this class
    const int val = p.mt == cls ? p.nb : 0;
    const int cs = wave_excl_scan_i32(val, lane);
    u64 segs = __ballot(val > 0 && cs < hi && cs + val > lo);
    const int64_t slot = (int64_t)h * P + y;
    while (segs) {
        const int b = (int)__builtin_ctzll(segs);
        segs &= segs - 1;
        const int csb = __builtin_amdgcn_readlane(cs, b), nbb = __builtin_amdgcn_readlane(val, b);
        const int kb0 = max(lo, csb) - csb, kb1 = min(hi, csb + nbb) - csb;
        TileDest dst;
        dst.direct = kb0 == 0 && kb1 == nbb;
        const int which = csb < lo ? 0 : 1;
        dst.o = part.o + (slot * 2 + which) * ATT_MTILE * D;
        dst.ml = part.ml + (slot * 2 + which) * ATT_MTILE;
        tile_segment<D>(a, s_dyn, h, b, tile * ATT_MTILE, kb0, kb1, dst);
    }
}

// Merge of the partials of the balanced schedule: one thread per (row, 4 output columns) of
// sequence blockIdx.y.  A sequence that stayed inside one gang was written directly.
template <int D>
__global__ __launch_bounds__(256) void attn_gang_combine_kernel(AttnArgs a, int P, GangPartial part) {
    const int b = blockIdx.y;
    const int *e = part.seq + b * GS_WORDS;
    const int jf = e[GS_FIRST], jl = e[GS_LAST];
    if (jf == jl) return;
    const int base = e[GS_BASE], cls = e[GS_CLS], Tc = e[GS_T], csb = e[GS_START];
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int G = a.Hq / a.Hkv;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int c4 = (int)(idx % (D / 4));
    const int64_t r = idx / (D / 4);  // row inside the sequence: node * Hq + head
    if (r >= (int64_t)N * a.Hq) return;
    const int node = (int)(r / a.Hq), hq = (int)(r % a.Hq), h = hq / G;
    const int mq = node * G + hq % G, tile = mq / ATT_MTILE, rit = mq % ATT_MTILE;
    const float c = a.scale * 1.4426950408889634f;
    auto prow = [&](int j) {
        const int64_t slot = (int64_t)h * P + base + j * cls + tile;
        return (slot * 2 + (csb < j * Tc ? 0 : 1)) * ATT_MTILE + rit;
    };
    // Four partials at a time, every load asked for before any is used (a load that waited for the
    // previous partial's weight would make the kernel one memory round trip per partial long); the
    // running maximum moves as in the attention kernel itself.
    float M = -INFINITY, l = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j0 = jf; j0 <= jl; j0 += 4) {
        float2 ml[4];
        float4 o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t pr = prow(min(j0 + u, jl));
            ml[u] = part.ml[pr];
            o[u] = *(const float4 *)(part.o + pr * D + c4 * 4);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (j0 + u > jl || !(ml[u].y > 0.f)) continue;  // a range whose keys were all hidden weighs nothing
            const float M2 = fmaxf(M, ml[u].x);
            const float keep = __builtin_amdgcn_exp2f((M - M2) * c);  // first partial: exp2(-inf) = 0
            const float wgt = __builtin_amdgcn_exp2f((ml[u].x - M2) * c);
            acc.x = acc.x * keep + o[u].x * wgt; acc.y = acc.y * keep + o[u].y * wgt;
            acc.z = acc.z * keep + o[u].z * wgt; acc.w = acc.w * keep + o[u].w * wgt;
            l = l * keep + ml[u].y * wgt;
            M = M2;
        }
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    bf16x4 o4;
    o4[0] = (__bf16)(acc.x * inv); o4[1] = (__bf16)(acc.y * inv);
    o4[2] = (__bf16)(acc.z * inv); o4[3] = (__bf16)(acc.w * inv);
    *(bf16x4 *)((__bf16 *)a.out + ((int64_t)b * a.TT_cap * a.Hq + r) * D + c4 * 4) = o4;
}

// ------------------------------------------------------------------- small-batch kernel -----
// When a batch offers only a few (sequence, kv head) pairs, latency matters more than reuse:
// one workgroup owns 32 query rows, its NW waves take the key blocks round-robin and stream
// them PRIVATELY (coalesced 16-byte loads, a wave-private LDS tile to bring K into operand
// layout and V into transposed operand layout, next block prefetched into registers), so the
// main loop has no barrier at all.  The partial results meet in LDS once at the end; nothing
// goes through global scratch.  Two variants: eight waves that stage each block through registers
// into padded tiles (one workgroup per unit, short key ranges), and four waves that load straight
// into LDS (DIRECT: several workgroups per unit, one wave per SIMD, so latency is hidden inside the
// wave by having every operand read of a block in flight at once).
#define KT_ELEMS (ATT_KB * K_PITCH)              // per-wave K tile: 32 rows of 272 B
#define WT_ELEMS (KT_ELEMS + ATT_KB * V_PITCH)   // both tiles of a wave (V: 32 rows of 288 B): 17.5 KB
#define WD_TILE (ATT_KB * 256)                  // direct layout: one K or V tile of a wave, unpadded rows
#define WD_STAGE (2 * WD_TILE)                  // K tile + V tile of one stage
#define WD_LDS_BYTES (4 * 2 * WD_STAGE)         // four waves, two stages: 128 KB

// With KS > 1 the key blocks are additionally dealt over KS workgroups per (sequence, kv head,
// row block); each leaves its partial (max, sum, O) in global scratch for a small merge kernel.
// (Merging in the last workgroup to arrive was tried: the device-scope release/acquire it needs
// writes back and invalidates the whole L2 of the XCD and cost far more than a second launch.)
struct SplitBuf {
    float4 *o;    // [unit, KS, 4 waves, 4, 64 lanes]: the owner waves' output registers
    float2 *ml;   // [unit, KS, 32]: (max, sum) per query row
};

template <int D, int NW, bool DIRECT>
__global__ __launch_bounds__(64 * NW) void attn_wave_kernel(AttnArgs a, int KS, SplitBuf sb) {
    static_assert(D == 128 && (NW == 4 || NW == 8) && (!DIRECT || NW == 4), "shape");
    constexpr int KSTEPS = D / 16, DBLK = D / 32;
    const int G = a.Hq / a.Hkv;
    // blockIdx.x = kv head: workgroups are dealt to the 8 XCDs round-robin by linear id, so every
    // row block and split of one kv head lands on one XCD and shares its L2 copy of that head's K/V
    const int b = blockIdx.z / KS, ks = blockIdx.z % KS, h = blockIdx.x;
    // the four per-sequence words, asked for together: one trip to memory instead of up to three
    const int n_raw = a.n_nodes[b], l_raw = a.prefix_len[b];
    const void *kp_raw = a.k_prefix[b], *vp_raw = a.v_prefix[b];
    const int N = min(max(n_raw, 1), a.TT_cap);
    const int M = N * G;
    const int m0 = blockIdx.y * 32;
    if (m0 >= M) return;
    const int L = max(l_raw, 0);
    const int Tk = L + N;
    const int nb = (Tk + ATT_KB - 1) / ATT_KB;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, known uniform
    const int half = lane >> 5, col = lane & 31;
    const int mq = m0 + col;
    const bool qvalid = mq < M;
    const int node = qvalid ? mq / G : 0;
    const int hq = h * G + (qvalid ? mq % G : 0);

    // LDS: NW private tiles during the loop, then the exchange area of the partial results
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    __shared__ float s_m[NW][32], s_l[NW][32];
    __bf16 *kt = (__bf16 *)s_dyn + w * WT_ELEMS;   // staged layout (!DIRECT): padded rows
    __bf16 *vt = kt + KT_ELEMS;
    unsigned char *wtile = s_dyn + w * 2 * WD_STAGE;  // direct layout: two stages of (K tile, V tile), 256-byte rows

    bf16x8 qreg[KSTEPS];
    {
        const __bf16 *qp = (const __bf16 *)a.q + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) qreg[s] = *(const bf16x8 *)(qp + 16 * s + 8 * half);  // rows past M read node 0: unused
    }
    const u64 mask0 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS];
    const u64 mask1 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS + 1];

    f32x16 oacc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale * 1.4426950408889634f;

    const gbf16p kpre = (gbf16p)kp_raw + (int64_t)h * a.kv_stride_head;
    const gbf16p vpre = (gbf16p)vp_raw + (int64_t)h * a.kv_stride_head;
    const gbf16p ktree = (gbf16p)a.k_tree + ((int64_t)b * a.TT_cap * a.Hkv + h) * D;
    const gbf16p vtree = (gbf16p)a.v_tree + ((int64_t)b * a.TT_cap * a.Hkv + h) * D;
    const int64_t stok = a.kv_stride_tok, stree = (int64_t)a.Hkv * D;
    const int kstep = KS * NW;  // the blocks are dealt round-robin over all waves of all splits
    if constexpr (DIRECT) {
        // Blocks go straight from global memory into the wave's own LDS tiles (global_load_lds_dwordx4:
        // the 64 x 16 B of one instruction land contiguously, i.e. four 256-byte rows), two stages, so
        // no staging registers and no LDS-write instructions; with one wave per SIMD the registers
        // saved are what lets every operand read of a block be in flight at once.  Chunk c of row r sits
        // at chunk position c ^ f(r), f as in the large-batch kernel, applied on the global side.
        const int krow4 = lane >> 4, cpos = lane & 15;
        u32 koffp[8], voffp[8];  // inside the prefix: byte offsets from the block's first row
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + krow4;
            koffp[i] = (u32)(r * stok + 8 * (cpos ^ (r & 15))) * 2u;
            voffp[i] = (u32)(r * stok + 8 * (cpos ^ (((r & 3) << 2) | ((r >> 2) & 3)))) * 2u;
        }
        const bool small_stride = (int64_t)ATT_KB * stok * 2 < ((int64_t)1 << 31);
        // Every load is unconditional: keys past the end are read from the last valid row, their scores
        // are masked to -inf below, so the duplicated V rows contribute nothing.
        auto fetch = [&](int kb, int stage) {
            const ldsp kdst = (ldsp)wtile + stage * WD_STAGE;
            const ldsp vdst = kdst + WD_TILE;
            if (small_stride && kb * ATT_KB + ATT_KB <= L) {  // block inside the prefix (uniform test)
                const gbytep kbase = (gbytep)(kpre + (int64_t)kb * ATT_KB * stok);
                const gbytep vbase = (gbytep)(vpre + (int64_t)kb * ATT_KB * stok);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    __builtin_amdgcn_global_load_lds(kbase + koffp[i], kdst + i * 1024, 16, 0, 0);
                    __builtin_amdgcn_global_load_lds(vbase + voffp[i], vdst + i * 1024, 16, 0, 0);
                }
            } else {                                           // block touching the tree keys or the end
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int r = 4 * i + krow4;
                    const int t = min(kb * ATT_KB + r, Tk - 1);
                    const int64_t o = t < L ? (int64_t)t * stok : (int64_t)(t - L) * stree;
                    __builtin_amdgcn_global_load_lds((gbytep)((t < L ? kpre : ktree) + o + 8 * (cpos ^ (r & 15))),
                                                     kdst + i * 1024, 16, 0, 0);
                    __builtin_amdgcn_global_load_lds(
                        (gbytep)((t < L ? vpre : vtree) + o + 8 * (cpos ^ (((r & 3) << 2) | ((r >> 2) & 3)))),
                        vdst + i * 1024, 16, 0, 0);
                }
            }
        };
        // operand read offsets (bytes inside a tile), as in the large-batch kernel
        u32 koff[KSTEPS];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) koff[s] = (u32)(col * 256 + (((2 * s + half) ^ (col & 15)) << 4));
        const int p16 = lane & 15, r0 = p16 >> 2, q4 = p16 & 3, grp = (lane >> 4) & 1;
        u32 voff[DBLK][2];
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi)
                voff[db][hi] = (u32)((8 * hi + 4 * half + r0) * 256 +
                                     (((4 * db + 2 * grp + (q4 >> 1)) ^ (4 * r0 + 2 * hi + half)) << 4) + 8 * (q4 & 1));

        int kb = ks * NW + w, cur = 0;
        if (kb < nb) fetch(kb, 0);
        for (; kb < nb; kb += kstep, cur ^= 1) {
            __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this block has landed
            if (kb + kstep < nb) fetch(kb + kstep, cur ^ 1);  // the other stage was last read one block ago
            const unsigned char *ktile = wtile + cur * WD_STAGE;  // K tile of this stage, its V tile behind it
            // Every operand of the block is asked for before it is needed (with one wave per SIMD nothing
            // else hides LDS latency): the eight K reads first, the sixteen transposing V reads between the
            // MFMAs of S^T, whose accumulator chain leaves the issue slots free.  K read s is followed by
            // 7 - s K reads and 2 s V reads when its MFMA comes up.
            const u32 kaddr = (u32)(uintptr_t)(ldsp)ktile, vaddr = kaddr + WD_TILE;
            bf16x8 ka[KSTEPS];
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) ka[s] = lds_load128(kaddr + koff[s]);
            bf16x4 vlo[DBLK][2], vhi[DBLK][2];
            f32x16 sacc;
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#define QK_STEP(s, db, st)                                                                  \
            lds_wait<7 + s>(ka[s]);                                                          \
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[s], sacc, 0, 0, 0);   \
            vlo[db][st] = lds_load_tr4<16 * st * 256>(vaddr + voff[db][0]);                  \
            vhi[db][st] = lds_load_tr4<16 * st * 256>(vaddr + voff[db][1]);                  \
            __builtin_amdgcn_sched_barrier(0);
            QK_STEP(0, 0, 0) QK_STEP(1, 1, 0) QK_STEP(2, 2, 0) QK_STEP(3, 3, 0)
            QK_STEP(4, 0, 1) QK_STEP(5, 1, 1) QK_STEP(6, 2, 1) QK_STEP(7, 3, 1)
#undef QK_STEP

            const int tbase = kb * ATT_KB;
            if (tbase + ATT_KB > L) {  // only blocks that contain tree keys (or the end) need the mask
                // 32-bit visibility window of this lane's query over keys tbase .. tbase+31: prefix keys
                // are visible, tree key j is visible iff bit j of the node's ancestor set (bits >= N are 0)
                const int off = tbase - L;  // uniform
                u32 vis;
                if (off >= 0) {
                    const u64 lo = off < 64 ? mask0 : mask1, hi = off < 64 ? mask1 : 0ull;
                    const int sh = off & 63;
                    vis = (u32)((lo >> sh) | (sh ? hi << (64 - sh) : 0ull));
                } else {
                    vis = ((u32)mask0 << (-off)) | ((1u << (-off)) - 1u);
                }
                vis >>= 4 * half;
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = ((vis >> (8 * (i >> 2) + (i & 3))) & 1u) ? sacc[i] : -INFINITY;
            }
            float mloc = sacc[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mloc = fmaxf(mloc, sacc[i]);
            mloc = half_swap_max(mloc);
            // lazily moved reference maximum, as in the large-batch kernel
            const bool move = (mloc - m_run) * c > LAZY_LOG2;
            const float m_new = move ? mloc : m_run;
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_use) * c) : 1.0f;
            const float nmc = -m_use * c;
            float psum = 0.f;
            bf16x8 pb[2];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, nmc));
                psum += p;
                pb[i >> 3][i & 7] = (__bf16)p;
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some query of this wave
#pragma unroll
                for (int db = 0; db < DBLK; ++db) acc_scale(oacc[db], alpha);
            }

            // All V reads have landed (they had the whole softmax).  The wait is tied to the very registers
            // the reads fill, and the halves are joined only behind it: a register copy made before the
            // data arrives would copy the old contents.  The "memory" clobber also keeps the next
            // iteration's loads into this stage behind this block's reads.
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(vlo[0][0]), "+v"(vhi[0][0]), "+v"(vlo[1][0]), "+v"(vhi[1][0]), "+v"(vlo[2][0]), "+v"(vhi[2][0]),
                           "+v"(vlo[3][0]), "+v"(vhi[3][0]), "+v"(vlo[0][1]), "+v"(vhi[0][1]), "+v"(vlo[1][1]), "+v"(vhi[1][1]),
                           "+v"(vlo[2][1]), "+v"(vhi[2][1]), "+v"(vlo[3][1]), "+v"(vhi[3][1])
                         :
                         : "memory");
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_shufflevector(vlo[db][st], vhi[db][st], 0, 1, 2, 3, 4, 5, 6, 7), pb[st], oacc[db], 0, 0, 0);
        }
    } else {
    const int kq = lane >> 4, dc = lane & 15;
    // Loading role of a lane, the same for K and V: load i takes key (i>>2)*16 + 4*kq + (i&3) of
    // the block, columns 8dc..8dc+7, so 16 lanes cover one 256-byte row (fully coalesced).
    // Inside the prefix the address is a uniform block base plus a fixed 32-bit lane offset.
    u32 loff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) loff[i] = (u32)(((i >> 2) * 16 + 4 * kq + (i & 3)) * stok + 8 * dc) * 2u;
    const bool small_stride = (int64_t)ATT_KB * stok * 2 < ((int64_t)1 << 31);

    // Every load is unconditional, so the sixteen loads of a block are in flight together.  Keys
    // past the end are read from the last valid row; their scores are masked to -inf below, so
    // their probabilities are exactly 0 and the duplicated V rows contribute nothing.
    bf16x8 kn[8], vn[8];
    auto fetch = [&](int kb) {
        if (small_stride && kb * ATT_KB + ATT_KB <= L) {  // block inside the prefix (uniform test)
            const gbytep kbase = (gbytep)(kpre + (int64_t)kb * ATT_KB * stok);
            const gbytep vbase = (gbytep)(vpre + (int64_t)kb * ATT_KB * stok);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                kn[i] = *(gbf16x8p)(kbase + loff[i]);
                vn[i] = *(gbf16x8p)(vbase + loff[i]);
            }
        } else {                                           // block touching the tree keys or the end
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int t = min(kb * ATT_KB + (i >> 2) * 16 + 4 * kq + (i & 3), Tk - 1);
                const int64_t o = (t < L ? (int64_t)t * stok : (int64_t)(t - L) * stree) + 8 * dc;
                kn[i] = gload8((t < L ? kpre : ktree) + o);
                vn[i] = gload8((t < L ? vpre : vtree) + o);
            }
        }
    };

    int kb = ks * NW + w;
    if (kb < nb) fetch(kb);
    for (; kb < nb; kb += kstep) {
        // The prefetched block goes straight into the wave's two LDS tiles, both row-major, which
        // frees its registers for the next prefetch, issued before any arithmetic on this block.
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = (i >> 2) * 16 + 4 * kq + (i & 3);
            *(bf16x8 *)(kt + r * K_PITCH + 8 * dc) = kn[i];
            *(bf16x8 *)(vt + r * V_PITCH + 8 * dc) = vn[i];
        }
        if (kb + kstep < nb) fetch(kb + kstep);

        f32x16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 ka = *(const bf16x8 *)(kt + col * K_PITCH + 16 * s + 8 * half);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc, 0, 0, 0);
        }

        const int tbase = kb * ATT_KB;
        if (tbase + ATT_KB > L) {  // only blocks that contain tree keys (or the end) need the mask
            // 32-bit visibility window of this lane's query over keys tbase .. tbase+31: prefix keys
            // are visible, tree key j is visible iff bit j of the node's ancestor set (bits >= N are 0)
            const int off = tbase - L;  // uniform
            u32 vis;
            if (off >= 0) {
                const u64 lo = off < 64 ? mask0 : mask1, hi = off < 64 ? mask1 : 0ull;
                const int sh = off & 63;
                vis = (u32)((lo >> sh) | (sh ? hi << (64 - sh) : 0ull));
            } else {
                vis = ((u32)mask0 << (-off)) | ((1u << (-off)) - 1u);
            }
            vis >>= 4 * half;
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[i] = ((vis >> (8 * (i >> 2) + (i & 3))) & 1u) ? sacc[i] : -INFINITY;
        }
        float mloc = sacc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mloc = fmaxf(mloc, sacc[i]);
        mloc = half_swap_max(mloc);
        // lazily moved reference maximum, as in the large-batch kernel
        const bool move = (mloc - m_run) * c > LAZY_LOG2;
        const float m_new = move ? mloc : m_run;
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_use) * c) : 1.0f;
        const float nmc = -m_use * c;
        float psum = 0.f;
        bf16x8 pb[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, nmc));
            psum += p;
            pb[i >> 3][i & 7] = (__bf16)p;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__ballot(alpha != 1.0f)) {  // the running maximum moved for some query of this wave
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }

        // O^T += V^T P^T.  The A operand of lane (column d = 32db + col, half) holds, for e = 0..7,
        // V[key 16st + 8(e/4) + 4half + e%4][d]: two transposing LDS reads of 4 keys each.  In a
        // 16-lane group lane p = 4j+q points at key j of the quadruple, columns d0 + 4q..4q+3.
        {
            const int p16 = lane & 15;
            const __bf16 *vbase = vt + (4 * half + (p16 >> 2)) * V_PITCH + 16 * ((lane >> 4) & 1) + 4 * (p16 & 3);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const bf16x4 lo = lds_read_tr4(vbase + (16 * st) * V_PITCH + 32 * db);
                    const bf16x4 hi = lds_read_tr4(vbase + (16 * st + 8) * V_PITCH + 32 * db);
                    const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[st], oacc[db], 0, 0, 0);
                }
        }
    }

    }

    // ---- the partial results meet ----------------------------------------------------------------
    float l_tot = half_swap_sum(l_run);
    __syncthreads();  // all private tiles are dead
    // exchange layout: float4 slot (slice, q, lane) at ((slice*16 + q)*64 + lane), q = 4 db + i/4
    float4 *xb = (float4 *)s_dyn;
    if (NW == 8) {
        // stage A: wave w+4 hands its whole partial to wave w
        if (w >= 4) {
            if (half == 0) { s_m[w][col] = m_run; s_l[w][col] = l_tot; }
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    xb[((w - 4) * 16 + db * 4 + q) * 64 + lane] =
                        make_float4(oacc[db][4 * q], oacc[db][4 * q + 1], oacc[db][4 * q + 2], oacc[db][4 * q + 3]);
        }
        __syncthreads();
        if (w < 4) {
            const float m2 = s_m[w + 4][col], l2 = s_l[w + 4][col];
            const float Mn = fmaxf(m_run, m2), Mu = Mn == -INFINITY ? 0.f : Mn;
            const float f1 = __builtin_amdgcn_exp2f((m_run - Mu) * c), f2 = __builtin_amdgcn_exp2f((m2 - Mu) * c);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 o = xb[(w * 16 + db * 4 + q) * 64 + lane];
                    oacc[db][4 * q] = oacc[db][4 * q] * f1 + o.x * f2;
                    oacc[db][4 * q + 1] = oacc[db][4 * q + 1] * f1 + o.y * f2;
                    oacc[db][4 * q + 2] = oacc[db][4 * q + 2] * f1 + o.z * f2;
                    oacc[db][4 * q + 3] = oacc[db][4 * q + 3] * f1 + o.w * f2;
                }
            l_tot = l_tot * f1 + l2 * f2;
            m_run = Mn;
        }
        __syncthreads();
    }
    // stage B: waves 0..3; wave w finishes output columns [32w, 32w+32)
    if (w < 4) {
        if (half == 0) { s_m[w][col] = m_run; s_l[w][col] = l_tot; }
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            if (db == w) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                xb[(w * 16 + db * 4 + q) * 64 + lane] =
                    make_float4(oacc[db][4 * q], oacc[db][4 * q + 1], oacc[db][4 * q + 2], oacc[db][4 * q + 3]);
        }
    }
    __syncthreads();
    if (w >= 4) return;
    float Mx = fmaxf(fmaxf(s_m[0][col], s_m[1][col]), fmaxf(s_m[2][col], s_m[3][col]));
    const float Mu = Mx == -INFINITY ? 0.f : Mx;
    float f[4], Lsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
        f[ww] = __builtin_amdgcn_exp2f((s_m[ww][col] - Mu) * c);
        Lsum += f[ww] * s_l[ww][col];
    }
    float res[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) res[i] = 0.f;
#pragma unroll
    for (int db = 0; db < DBLK; ++db)  // own block (db == w) from registers; static indexing only
        if (db == w)
#pragma unroll
            for (int i = 0; i < 16; ++i) res[i] = oacc[db][i] * f[db];
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
        if (ww == w) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 o = xb[(ww * 16 + w * 4 + q) * 64 + lane];
            res[4 * q] += o.x * f[ww];
            res[4 * q + 1] += o.y * f[ww];
            res[4 * q + 2] += o.z * f[ww];
            res[4 * q + 3] += o.w * f[ww];
        }
    }
    if (KS > 1) {
        // ---- leave this workgroup's partial for the merge kernel ---------------------------------
        const int64_t unit = ((int64_t)b * a.Hkv + h) * gridDim.y + blockIdx.y;
        float4 *pw = sb.o + ((unit * KS + ks) * 4 + w) * 4 * 64;
#pragma unroll
        for (int q = 0; q < 4; ++q) pw[q * 64 + lane] = make_float4(res[4 * q], res[4 * q + 1], res[4 * q + 2], res[4 * q + 3]);
        if (w == 0 && half == 0) sb.ml[(unit * KS + ks) * 32 + col] = make_float2(Mx, Lsum);
        return;
    }
    if (!qvalid) return;
    const float inv = Lsum > 0.f ? 1.0f / Lsum : 0.f;
    __bf16 *op = (__bf16 *)a.out + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D + 32 * w;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(res[q4 * 4 + e] * inv);
        *(bf16x4 *)(op + 8 * q4 + 4 * half) = o4;
    }
}

// Merge of the KS partials of every (sequence, kv head, 32-row block): thread (w, lane) owns the
// same 16 output values it would own in the single-split epilogue, so the partials are read
// back in exactly the layout they were written in.
template <int D>
__global__ __launch_bounds__(256) void attn_wave_merge_kernel(AttnArgs a, int KS, SplitBuf sb) {
    const int G = a.Hq / a.Hkv;
    const int b = blockIdx.z, h = blockIdx.x;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    const int M = N * G;
    const int m0 = blockIdx.y * 32;
    if (m0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int mq = m0 + col;
    if (mq >= M) return;
    const int node = mq / G, hq = h * G + mq % G;
    const float c = a.scale * 1.4426950408889634f;
    const int64_t unit = ((int64_t)b * a.Hkv + h) * gridDim.y + blockIdx.y;
    float Mall = -INFINITY;
    for (int s2 = 0; s2 < KS; ++s2) Mall = fmaxf(Mall, sb.ml[(unit * KS + s2) * 32 + col].x);
    const float Ma = Mall == -INFINITY ? 0.f : Mall;
    float res[16], Lsum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) res[i] = 0.f;
    for (int s2 = 0; s2 < KS; ++s2) {
        const float2 ml = sb.ml[(unit * KS + s2) * 32 + col];
        const float fs = __builtin_amdgcn_exp2f((ml.x - Ma) * c);
        Lsum += ml.y * fs;
        const float4 *pr = sb.o + ((unit * KS + s2) * 4 + w) * 4 * 64;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 o = pr[q * 64 + lane];
            res[4 * q] += o.x * fs;
            res[4 * q + 1] += o.y * fs;
            res[4 * q + 2] += o.z * fs;
            res[4 * q + 3] += o.w * fs;
        }
    }
    const float inv = Lsum > 0.f ? 1.0f / Lsum : 0.f;
    __bf16 *op = (__bf16 *)a.out + (((int64_t)b * a.TT_cap + node) * a.Hq + hq) * D + 32 * w;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(res[q4 * 4 + e] * inv);
        *(bf16x4 *)(op + 8 * q4 + 4 * half) = o4;
    }
}

// ------------------------------------------------------------------------------ fp32 path --
// One wave per (node, head).  Keys are taken 64 at a time: lane j scores key j, the wave
// agrees on the running maximum, then lane c accumulates output columns c, c+64.
template <typename T>
__device__ __forceinline__ float ld(const T *p);
template <>
__device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <>
__device__ __forceinline__ float ld<uint16_t>(const uint16_t *p) { return bf16_bits_to_float(*p); }

template <typename T>
__global__ __launch_bounds__(64) void attn_simple_kernel(AttnArgs a) {
    const int node = blockIdx.x, hq = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int N = min(max(a.n_nodes[b], 1), a.TT_cap);
    if (node >= N) return;
    const int D = a.D, G = a.Hq / a.Hkv, h = hq / G;
    const int L = max(a.prefix_len[b], 0), Tk = L + N;
    const int64_t row = ((int64_t)b * a.TT_cap + node) * a.Hq + hq;
    const T *q = (const T *)a.q + row * D;
    const T *kpre = (const T *)a.k_prefix[b], *vpre = (const T *)a.v_prefix[b];
    const T *ktree = (const T *)a.k_tree + (int64_t)b * a.TT_cap * a.Hkv * D;
    const T *vtree = (const T *)a.v_tree + (int64_t)b * a.TT_cap * a.Hkv * D;
    const u64 mask0 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS];
    const u64 mask1 = a.anc_mask[((int64_t)b * a.TT_cap + node) * DT_MASK_WORDS + 1];

    __shared__ float s_q[128];
    for (int cidx = lane; cidx < D; cidx += 64) s_q[cidx] = ld(q + cidx);
    __syncthreads();

    float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;
    for (int t0 = 0; t0 < Tk; t0 += 64) {
        const int t = t0 + lane;
        bool vis = t < Tk;
        if (vis && t >= L) {
            const int j = t - L;
            vis = ((j < 64 ? mask0 : mask1) >> (j & 63)) & 1ull;
        }
        float s = -INFINITY;
        if (vis) {
            const T *kp = t < L ? kpre + (int64_t)t * a.kv_stride_tok + (int64_t)h * a.kv_stride_head
                                : ktree + ((int64_t)(t - L) * a.Hkv + h) * D;
            // four partial sums, 64 loads requested together: the row is read at memory latency once per
            // 64 elements, not once per element
            float d4[4] = {0.f, 0.f, 0.f, 0.f};
            int cidx = 0;
            for (; cidx + 64 <= D; cidx += 64) {
                float kv[64];
#pragma unroll
                for (int u = 0; u < 64; ++u) kv[u] = ld(kp + cidx + u);
                __builtin_amdgcn_sched_barrier(0);  // all requests before the first use
#pragma unroll
                for (int u = 0; u < 64; ++u) d4[u & 3] = fmaf(s_q[cidx + u], kv[u], d4[u & 3]);
            }
            for (; cidx < D; ++cidx) d4[0] = fmaf(s_q[cidx], ld(kp + cidx), d4[0]);
            s = ((d4[0] + d4[1]) + (d4[2] + d4[3])) * a.scale;
        }
        const float m_new = fmaxf(m_run, wave_max(s));
        if (m_new == -INFINITY) continue;
        const float alpha = __expf(m_run - m_new);
        const float p = vis ? __expf(s - m_new) : 0.f;
        l_run = l_run * alpha + wave_sum(p);
        o0 *= alpha; o1 *= alpha;
        m_run = m_new;
        // V rows sixteen at a time, all their loads requested before the first is used; keys past the end
        // repeat the last row with probability 0
        const int cnt = min(64, Tk - t0);
        for (int j0 = 0; j0 < cnt; j0 += 16) {
            float v0[16], v1[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int tj = min(t0 + j0 + u, Tk - 1);
                const T *vp = tj < L ? vpre + (int64_t)tj * a.kv_stride_tok + (int64_t)h * a.kv_stride_head
                                     : vtree + ((int64_t)(tj - L) * a.Hkv + h) * D;
                v0[u] = ld(vp + min(lane, D - 1));        // unconditional (columns past D repeat the last one and
                v1[u] = ld(vp + min(lane + 64, D - 1));   // are never stored): a load in a branch is waited for there
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const float pj = __shfl(p, j0 + u, 64);  // lanes at and past cnt hold 0
                o0 = pj != 0.f ? fmaf(pj, v0[u], o0) : o0;   // a hidden key's row is not even multiplied by 0
                o1 = pj != 0.f ? fmaf(pj, v1[u], o1) : o1;
            }
        }
    }
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
    if (sizeof(T) == 4) {
        float *op = (float *)a.out + row * D;
        if (lane < D) op[lane] = o0 * inv;
        if (lane + 64 < D) op[lane + 64] = o1 * inv;
    } else {
        __bf16 *op = (__bf16 *)a.out + row * D;
        if (lane < D) op[lane] = (__bf16)(o0 * inv);
        if (lane + 64 < D) op[lane + 64] = (__bf16)(o1 * inv);
    }
}

// ------------------------------------------------------------------------------- launchers --
// LDS beyond 64 KB has to be asked for, once per device (dt_init)
hipError_t attn_init() {
    hipError_t e = hipFuncSetAttribute((const void *)attn_wave_kernel<128, 8, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       8 * WT_ELEMS * 2);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)attn_wave_kernel<128, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                WD_LDS_BYTES);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)attn_tile_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, TILE_LDS_BYTES);
    if (e == hipSuccess)
        e = hipFuncSetAttribute((const void *)attn_gang_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, TILE_LDS_BYTES);
    return e;
}

// scratch of the balanced large-batch schedule: (kv heads x slots per head) <= 2 x compute units
// slots, two partials of 128 rows each, and the table of up to 64 sequences
static size_t gang_bytes(int D, int n_cu) {
    return (size_t)2 * n_cu * 2 * ATT_MTILE * ((size_t)D * 4 + 8) + 64 * GS_WORDS * 4;
}

// scratch of the small-batch key splits: per (sequence, kv head, 32-row block) and split
static size_t wave_split_bytes(int batch, int TT_cap, int Hq) {
    return (size_t)batch * ((TT_cap * Hq + 31) / 32 + Hq) * (4 * 4 * 64 * 16 + 32 * 8);
}

size_t attn_workspace_bytes(int batch, int TT_cap, int Hq, int D, int n_cu) {
    if (D != 128) return 0;
    const size_t w8 = wave_split_bytes(batch, TT_cap, Hq) * 8, g = gang_bytes(D, n_cu);
    const size_t cap = (size_t)256 << 20;
    const size_t want = w8 > g ? w8 : g;
    return want < cap ? want : cap;
}

int attn_launch(const AttnArgs &a, hipStream_t st, hipError_t *err) {
    *err = hipSuccess;
    if (a.batch <= 0) return DT_OK;
    const bool mfma = a.dtype == DT_BF16 && a.D == 128 && a.kv_stride_tok % 8 == 0 && a.kv_stride_head % 8 == 0;
    if (!mfma) {
        if (a.D > 128) return DT_ERR_LIMIT;
        dim3 grid(a.TT_cap, a.Hq, a.batch);
        if (a.dtype == DT_BF16) launch_kernel(KID_ATTN, st, attn_simple_kernel<uint16_t>, grid, dim3(64), 0, a);
        else launch_kernel(KID_ATTN, st, attn_simple_kernel<float>, grid, dim3(64), 0, a);
        *err = hipGetLastError();
        return *err == hipSuccess ? DT_OK : DT_ERR_HIP;
    }
    const int G = a.Hq / a.Hkv;
    const int mtiles = (a.TT_cap * G + ATT_MTILE - 1) / ATT_MTILE;
    const int base_wgs = a.batch * a.Hkv * mtiles;
    if (base_wgs < 128) {
        // few (sequence, kv head, row tile) items: the barrier-free small-batch kernel
        // Key splits: towards one workgroup per compute unit, but only while a split still owns
        // about 20 key blocks -- below that the fixed cost of a workgroup (query load, first
        // fetch, LDS exchange) plus the merge launch outweighs the shorter loop (measured).
        const int mblocks = (a.TT_cap * G + 31) / 32;
        const int units = a.batch * a.Hkv * mblocks;
        const int nb_max = (a.max_prefix_len + a.TT_cap + ATT_KB - 1) / ATT_KB;
        int KS = 256 / units;
        if (KS > 8) KS = 8;
        if (KS > nb_max / 11) KS = nb_max / 11;
        const size_t per_split = (size_t)units * (4 * 4 * 64 * 16 + 32 * 8);
        if (KS > 1 && (!a.ws || (size_t)KS * per_split > a.ws_bytes)) KS = a.ws ? (int)(a.ws_bytes / per_split) : 1;
        if (KS < 1) KS = 1;
        int nw_sel = KS > 1 ? 4 : 8;
        SplitBuf sb;
        sb.o = (float4 *)a.ws;
        sb.ml = (float2 *)((char *)a.ws + (size_t)units * KS * 4 * 4 * 64 * 16);
        dim3 grid(a.Hkv, mblocks, a.batch * KS);
        if (nw_sel == 4)  // several workgroups per unit: four waves each, one workgroup per compute unit (128 KB of LDS)
            launch_kernel(KID_ATTN, st, attn_wave_kernel<128, 4, true>, grid, dim3(256), WD_LDS_BYTES, a, KS, sb);
        else              // one workgroup per unit: eight waves (two per SIMD), 136 KB of LDS
            launch_kernel(KID_ATTN, st, attn_wave_kernel<128, 8, false>, grid, dim3(512), 8 * WT_ELEMS * 2, a, KS, sb);
        if (KS > 1) {
            *err = hipGetLastError();
            if (*err != hipSuccess) return DT_ERR_HIP;
            launch_kernel(KID_ATTN_COMBINE, st, attn_wave_merge_kernel<128>, dim3(a.Hkv, mblocks, a.batch), dim3(256), 0,
                          a, KS, sb);
        }
        *err = hipGetLastError();
        return *err == hipSuccess ? DT_OK : DT_ERR_HIP;
    }
    // Fewer whole (sequence, kv head, row tile) items than four rounds of two workgroups per compute
    // unit: the balanced schedule (needs one lane per sequence and a slot for every tile count).
    const int P = 2 * a.n_cu / a.Hkv;
    const bool gang = base_wgs < 8 * a.n_cu && a.batch <= 64 && mtiles <= 63 && P >= mtiles * (mtiles + 1) / 2 &&
                      a.ws && (size_t)a.Hkv * P * 2 * ATT_MTILE * ((size_t)a.D * 4 + 8) + 64 * GS_WORDS * 4 <= a.ws_bytes;
    if (!gang) {
        launch_kernel(KID_ATTN, st, attn_tile_kernel<128>, dim3(a.Hkv, mtiles, a.batch), dim3(256), TILE_LDS_BYTES, a);
        *err = hipGetLastError();
        return *err == hipSuccess ? DT_OK : DT_ERR_HIP;
    }
    GangPartial part;
    part.o = (float *)a.ws;
    part.ml = (float2 *)((char *)a.ws + (size_t)a.Hkv * P * 2 * ATT_MTILE * a.D * 4);
    part.seq = (int *)((char *)a.ws + (size_t)a.Hkv * P * 2 * ATT_MTILE * ((size_t)a.D * 4 + 8));
    launch_kernel(KID_ATTN, st, attn_gang_kernel<128>, dim3(a.Hkv, P), dim3(256), TILE_LDS_BYTES, a, P, mtiles, part);
    *err = hipGetLastError();
    if (*err != hipSuccess) return DT_ERR_HIP;
    const int64_t items = (int64_t)a.TT_cap * a.Hq * (a.D / 4);
    launch_kernel(KID_ATTN_COMBINE, st, attn_gang_combine_kernel<128>, dim3((unsigned)((items + 255) / 256), a.batch),
                  dim3(256), 0, a, P, part);
    *err = hipGetLastError();
    return *err == hipSuccess ? DT_OK : DT_ERR_HIP;
}

}  // namespace dt
