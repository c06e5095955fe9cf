// FlashAttention forward for gfx950 with a selectable K/V scan order (cyclic or sawtooth).
//
// One workgroup = 4 wavefronts = one 128-row query tile (paper Sec. 2.2, Alg. 1); wavefront w owns
// query rows 32w..32w+31 of the tile and keeps them in registers for the whole inner loop.  K and V
// are streamed in 64-row tiles through two LDS buffers each, filled by direct global->LDS loads.
//
// Both contractions run on v_mfma_f32_32x32x16 in the transposed form
//     S^T (kv x q) = K_j   (kv x d) . Q_i^T (d x q)
//     O^T (d  x q) = V_j^T (d x kv) . P^T   (kv x q)
// because the accumulator layout of S^T (a lane holds, for its query column lane%32, the kv rows
// 8*(r/4) + 4*(lane/32) + r%4 of a 32-row block in register r) is, register for register, the
// B-operand layout of the second product once the contraction index of each 16-wide MFMA step is
// read as  slot (lane/32, e) <-> kv = 16*step + 8*(e/4) + 4*(lane/32) + e%4.  So P never leaves
// registers.  V^T in the matching A-operand layout comes from ds_read_b64_tr_b16, which hands lane
// i of a 16-lane group the column i of a 4 x 16 block whose four row addresses are supplied by
// lanes 4e + c (row e, 8-byte column chunk c) of that group.
//
// Softmax statistics live per lane: lanes l and l+32 share a query row and hold disjoint key
// subsets, so the running maximum is merged across the pair every tile while the running sum stays
// a per-lane partial (it is linear) and is merged once in the epilogue.
//
// A query tile's scan is a software-pipelined run of full, unmasked K/V tiles (pipelined_range)
// plus, at one end, a short run of masked tiles (general_range).  The workgroups of one XCD walk
// the same head together and re-align between heads (domain_sync).
//
// For head dimension 128 there is a second tile shape (NH = 2 in the templates, pipelined_range_wide):
// a wavefront owns two such 32-row halves, a workgroup 256 query rows, one workgroup per CU, and every
// K / V^T fragment read from LDS feeds one MFMA per half.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <type_traits>
#include <utility>

#include "sawattn.h"
#include "schedule.h"

// Scratch memory of attn_fwd_static (the entry point that may not allocate): binary16 copies of K and V.
// In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[SAWATTN_STATIC_SCRATCH_BYTES];

namespace sawattn {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef __bf16 b4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u16v __attribute__((ext_vector_type(16)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*

struct Params {
    const void* Q;
    const void* K;
    const void* V;
    void* O;
    int32_t* trace;        // optional: [grid][max_local][4]
    int32_t* trace_count;  // optional: [grid]
    int N;
    int o_dtype;
    int sawtooth;
    int negate_q;          // scale < 0: use -Q and |scale|
    int q_bf16;            // wide variant on converted inputs: Q is still bfloat16 (K and V are binary16 copies)
    int stream_o;          // O leaves through LDS as whole lines, non-temporal (variant.qo_streaming)
    int stream_q;          // Q arrives through LDS as whole lines, non-temporal
    int max_local;
    int ticket_set;        // which set of arrival counters this launch uses (domain_sync)
    float c;               // |scale| * log2(e): scores are handled in the log2 domain
    Schedule sched;
};

// LDS tile layout.  A tile is 64 rows of D 16-bit elements, rows packed back to back (no padding, so
// that one wavefront-wide direct global->LDS load, which writes 64 x 16 contiguous bytes, fills whole
// rows).  Inside a row the 16-byte chunks are permuted: chunk cc of row r sits at chunk position
// cc ^ swz(r).  swz is chosen so that both read patterns are free of bank conflicts:
//   * K operand: 16 lanes read the same chunk of 16 consecutive rows          -> swz distinct over them
//   * V operand (ds_read_b64_tr_b16): 32 lanes read 4 consecutive rows x 64 B -> the rows land in
//     four different 64-byte bank groups.
template <int D>
struct Geo {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;                       // 16-byte chunks per row
    static constexpr int kTile = kTileKV * kRowBytes;                 // one K or V tile in LDS
    static constexpr int kRowsPerWaveLoad = 1024 / kRowBytes;         // rows one 64-lane x 16 B load covers
    static constexpr int kLoadsPerWave = kTile / 1024 / (kThreads / 64);
    static constexpr int kLdsBytes = 4 * kTile;                       // K0 K1 V0 V1
    __device__ static __forceinline__ int swz(int row) {
        if constexpr (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
        else return ((row & 2) << 1) | ((row >> 2) & 3);              // u = row>>1: (u&1)<<2 | (u>>1)&3
    }
};

template <bool BF16>
__device__ __forceinline__ f16v mfma_16bit(u4 a, u4 b, f16v c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

// Eight bfloat16 -> eight binary16 (round to nearest even; exact for normal binary16 magnitudes).
__device__ __forceinline__ u4 bf16x8_to_f16x8(u4 w) {
    u4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f2 x;
        x[0] = __builtin_bit_cast(float, w[i] << 16);
        x[1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
        r[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(x, h2));
    }
    return r;
}

// Compile-time loop: f(std::integral_constant<int, I>) for I in [0, N).
template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl<N>(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// Lane-constant addresses, computed once per kernel.
//
// Tile fill: wavefront w, load i covers LDS bytes [(i*4 + w) * 1024, +1024) of a tile: lane l
// writes chunk position l % CPR of row (i*4+w)*rows_per_load + l / CPR and therefore fetches source
// chunk (l % CPR) ^ swz(row) of that row.
// K operand (S^T = K Q^T): lane reads chunk 2*ks + g of rows ln and 32 + ln (same swz for both).
// V operand (ds_read_b64_tr_b16): source lane 4e + c of a 16-lane group addresses row e, 8-byte
// column chunk c of the 4 x 16 block whose columns the lanes of the group receive; the rows are
// kv = 16*ks + 8*h + 4*g + e, so that the contraction slots line up with the registers of P^T.
template <int D>
struct LaneMap {
    using G = Geo<D>;
    unsigned fill_src[G::kLoadsPerWave];   // row * row_bytes + byte offset of the source chunk
    unsigned fill_dst;                     // wave * 1024 (+ i * 4096): LDS byte offset inside the tile
    unsigned k_rd[D / 16];                 // byte offset inside a K tile, MFMA step ks, rows ln (+32 rows: +32*row_bytes)
    unsigned v_rd[D / 32][2];              // byte offset inside a V tile for [db][h], kv step 0 (+ks: +16*row_bytes*ks)
    __device__ __forceinline__ LaneMap(int wave, int lane) {
        const int g = lane >> 5, ln = lane & 31;
#pragma unroll
        for (int i = 0; i < G::kLoadsPerWave; ++i) {
            const int r = (i * 4 + wave) * G::kRowsPerWaveLoad + lane / G::kChunksPerRow;
            fill_src[i] = r * G::kRowBytes + ((lane % G::kChunksPerRow) ^ G::swz(r)) * 16;
        }
        fill_dst = wave * 1024;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) k_rd[ks] = ln * G::kRowBytes + ((2 * ks + g) ^ G::swz(ln)) * 16;
        const int vrow = 4 * g + ((lane & 15) >> 2);
        const int chunk = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        const int half = (lane & 1) * 8;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = vrow + 8 * h;     // swz(r + 16*ks) == swz(r)
                v_rd[db][h] = r * G::kRowBytes + ((4 * db + chunk) ^ G::swz(r)) * 16 + half;
            }
    }
};

// One 64-lane x 16-byte direct global -> LDS load: lane l's 16 bytes from base + voff land at LDS
// byte address lds_addr + 16*l.  Issued as inline assembly so that the compiler does not treat every
// later LDS read as depending on it (it would wait for the whole next tile before reading the
// current one); the landing is awaited explicitly with wait_tile_landed() before the barrier that
// publishes the tile.
__device__ __forceinline__ void load_to_lds_16B(const char* base, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}
// The same marked non-temporal: data read once (a Q tile) that should not take the place of K/V tiles in the L2.
__device__ __forceinline__ void load_to_lds_16B_nt(const char* base, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}
// The same with the LDS address given as a scalar base plus a compile-time offset (one scalar add into M0).
template <int LDS_IMM>
__device__ __forceinline__ void load_to_lds_16B_at(const char* base, unsigned voff, unsigned lds_base) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(voff), "s"(base), "n"(LDS_IMM) : "memory", "m0", "scc");
}
__device__ __forceinline__ void wait_tile_landed() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Per-lane byte offsets (relative to the head's base) of this lane's chunks of tile j.  A ragged
// last tile re-reads row N-1 for the rows beyond N: always valid memory and finite data; such
// keys are masked before use.
template <int D>
__device__ __forceinline__ void tile_offsets(int j, int N, const LaneMap<D>& lm, unsigned (&off)[Geo<D>::kLoadsPerWave]) {
    using G = Geo<D>;
    const int kv0 = j * kTileKV;
    if (kv0 + kTileKV <= N) {
#pragma unroll
        for (int i = 0; i < G::kLoadsPerWave; ++i) off[i] = lm.fill_src[i];
    } else {
#pragma unroll
        for (int i = 0; i < G::kLoadsPerWave; ++i) {
            const unsigned row = lm.fill_src[i] / G::kRowBytes, chunk = lm.fill_src[i] % G::kRowBytes;
            unsigned r = kv0 + row;
            r = r < (unsigned)N ? r : (unsigned)N - 1;
            off[i] = (r - kv0) * G::kRowBytes + chunk;   // (r >= kv0: tile j exists, so its first row is below N)
        }
    }
}

// Direct global -> LDS copy of tile j of a head into the tile at LDS byte address dst.
template <int D>
__device__ __forceinline__ void tile_to_lds(const char* head, int j, const unsigned (&off)[Geo<D>::kLoadsPerWave],
                                            const LaneMap<D>& lm, unsigned dst) {
    using G = Geo<D>;
    const char* base = head + (size_t)j * kTileKV * G::kRowBytes;
#pragma unroll
    for (int i = 0; i < G::kLoadsPerWave; ++i) load_to_lds_16B(base, off[i], dst + lm.fill_dst + i * 4096);
}

// Register path for V in bfloat16 (converted to binary16 before it reaches LDS).
template <int D>
__device__ __forceinline__ void tile_to_regs(const char* head, int j, const unsigned (&off)[Geo<D>::kLoadsPerWave],
                                             u4 (&reg)[Geo<D>::kLoadsPerWave]) {
    using G = Geo<D>;
    const char* base = head + (size_t)j * kTileKV * G::kRowBytes;
#pragma unroll
    for (int i = 0; i < G::kLoadsPerWave; ++i) reg[i] = *reinterpret_cast<const u4*>(base + off[i]);
}
template <int D>
__device__ __forceinline__ void regs_to_lds_f16(const u4 (&reg)[Geo<D>::kLoadsPerWave], const LaneMap<D>& lm, int lane,
                                                LDS_PTR(char) dst) {
    using G = Geo<D>;
#pragma unroll
    for (int i = 0; i < G::kLoadsPerWave; ++i)
        *(LDS_PTR(u4))(dst + lm.fill_dst + i * 4096 + lane * 16) = bf16x8_to_f16x8(reg[i]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between the lanes l and l^32, the two lanes that share a query row.  v_permlane32_swap
// swaps the upper 32 lanes of its first operand with the lower 32 lanes of its second; starting
// from two copies of x this leaves (lower half of x everywhere, upper half of x everywhere).
__device__ __forceinline__ void lane_pair(float x, float& lower, float& upper) {
    unsigned a = __builtin_bit_cast(unsigned, x), b = a;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    lower = __builtin_bit_cast(float, a);
    upper = __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float pair_max(float x) {
    float lo, hi;
    lane_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float pair_sum(float x) {
    float lo, hi;
    lane_pair(x, lo, hi);
    return lo + hi;
}

// Adds the two binary16 values of `ph` to two float partial sums (one mixed-precision FMA each:
// exact, and cheaper in the instruction stream than the two-element dot product).
// `one` is binary16 1.0 held in a register the compiler cannot see through (opaque_one()): the widened products
// then become v_fma_mix_f32.  Written in C and not as inline assembly because the compiler separates dependent
// assembly statements that have nothing in between by a no-op each, one issue slot per row-sum update.
__device__ __forceinline__ _Float16 opaque_one() {
    _Float16 one = (_Float16)1.0f;
    asm volatile("" : "+v"(one));
    return one;
}
__device__ __forceinline__ void add_pair(float& sum_lo, float& sum_hi, h2 ph, _Float16 one) {
    sum_lo = __builtin_fmaf((float)ph[0], (float)one, sum_lo);
    sum_hi = __builtin_fmaf((float)ph[1], (float)one, sum_hi);
}

// The running maximum is only raised when a tile's maximum exceeds it by more than this many
// binades; until then probabilities are taken relative to the older, smaller reference and may be
// as large as 2^kRescaleSlack.  O and the running sum stay consistent, so the result is unchanged;
// it saves rescaling the whole accumulator on almost every tile.
constexpr float kRescaleSlack = 8.0f;

// Per-wavefront state of one query tile that the K/V loop carries along.
template <int D>
struct TileState {
    u4 qf[D / 16];      // Q^T as B operand: lane holds Q[qrow][16*ks + 8*g .. +7]
    f16v o[D / 32];     // O^T accumulator
    float M;            // reference maximum of score*c (log2 domain), same in both lanes of a pair
    float L;            // this lane's partial running sum
};

// This lane's LDS read addresses for the K/V buffer pair in use; flipped to the other pair after
// every iteration.
template <int D>
struct ReadAddr {
    unsigned k[D / 16];       // K operand, MFMA step ks, row ln (+32 rows: +32*row_bytes)
    unsigned v[D / 32][2];    // V operand [db][h], kv step 0 (+ks: +16*row_bytes*ks)
    __device__ __forceinline__ void flip(int delta) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) k[ks] += delta;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) { v[db][0] += delta; v[db][1] += delta; }
    }
};

// MFMAs of the wide variant, written out so that the register file of every operand is fixed: with
// more than 256 registers per wavefront the accumulation registers (AccVGPRs) have to hold what only
// the matrix pipe touches -- the O^T accumulators and the Q^T fragments -- and nothing the vector ALU
// reads, or every use costs a copy.  The compiler does not see these as MFMAs and inserts no wait
// states for them; mfma_settle_*() is placed wherever the vector ALU reads an accumulator that the
// few preceding instructions may still be writing (8 passes + 3 wait states).
template <bool BF16>
__device__ __forceinline__ void mfma_s_first(f16v& acc, u4 k_frag, const u4& q_frag) {
    if constexpr (BF16) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(k_frag), "a"(q_frag));
    else asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(acc) : "v"(k_frag), "a"(q_frag));
}
template <bool BF16>
__device__ __forceinline__ void mfma_s(f16v& acc, u4 k_frag, const u4& q_frag) {
    if constexpr (BF16) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(k_frag), "a"(q_frag));
    else asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(k_frag), "a"(q_frag));
}
__device__ __forceinline__ void mfma_o(f16v& acc, s8 v_frag, const u4& p_frag) {
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(v_frag), "v"(p_frag));
}
// The accumulators pass through the statement, so that no use of them can be scheduled ahead of it.
__device__ __forceinline__ void mfma_settle_v(f16v& a0, f16v& a1, f16v& a2, f16v& a3) {
    asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));
}
__device__ __forceinline__ void mfma_settle_v(f16v& a0, f16v& a1) {
    asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a0), "+v"(a1));
}
template <int NACC>
__device__ __forceinline__ void mfma_settle_a(f16v (&acc)[NACC]) {
    asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");
#pragma unroll
    for (int i = 0; i < NACC; ++i) asm volatile("" : "+a"(acc[i]));
}
// The other direction: accumulators that vector instructions (or the compiler's copies into accumulation
// registers) may just have written are placed in their register file here, and the MFMAs that read them
// start a few wait states later.
template <int NACC>
__device__ __forceinline__ void mfma_guard(f16v (&acc)[NACC]) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) asm volatile("" : "+a"(acc[i]));
    asm volatile("s_nop 7" ::: "memory");
}

// One K/V tile for one wavefront out of the LDS buffers `ra` points at: S^T = K Q^T, softmax
// update, O^T += V^T P^T.
// WIDE: the tile state is the wide variant's -- Q^T fragments and O^T accumulators live in accumulation
// registers and the MFMAs are the written-out ones.
template <int D, bool BF16, bool CAUSAL, bool MASKED, bool WIDE = false>
__device__ __forceinline__ void compute_tile(TileState<D>& st, const ReadAddr<D>& ra, float c, int kv0, int qrow, int lane,
                                             int N) {
    using G = Geo<D>;
    constexpr int KS = D / 16, DB = D / 32;
    const int g = lane >> 5;
    // ---- S^T = K_j Q_i^T : two 32(kv) x 32(q) blocks; operands fetched two steps ahead
    f16v s[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[0][r] = 0.f; s[1][r] = 0.f; }
    {
        u4 a[KS][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            a[ks][0] = *(LDS_PTR(u4))(size_t)(ra.k[ks]);
            a[ks][1] = *(LDS_PTR(u4))(size_t)(ra.k[ks] + 32 * G::kRowBytes);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 2 < KS) {
                a[ks + 2][0] = *(LDS_PTR(u4))(size_t)(ra.k[ks + 2]);
                a[ks + 2][1] = *(LDS_PTR(u4))(size_t)(ra.k[ks + 2] + 32 * G::kRowBytes);
            }
            if constexpr (WIDE) {
                if (ks == 0) {
                    mfma_s_first<BF16>(s[0], a[ks][0], st.qf[ks]);
                    mfma_s_first<BF16>(s[1], a[ks][1], st.qf[ks]);
                } else {
                    mfma_s<BF16>(s[0], a[ks][0], st.qf[ks]);
                    mfma_s<BF16>(s[1], a[ks][1], st.qf[ks]);
                }
            } else {
                s[0] = mfma_16bit<BF16>(a[ks][0], st.qf[ks], s[0]);
                s[1] = mfma_16bit<BF16>(a[ks][1], st.qf[ks], s[1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (WIDE) mfma_settle_v(s[0], s[1]);
    }
    // ---- mask: keys at or beyond N, and keys after the query under the causal mask, get the score -inf, which
    //      c > 0 turns into the probability 0.  Register r of block b is key 32b + 8(r/4) + 4g + r%4 of the tile:
    //      visible up to the offset `ahead` (one comparison and one select per score).
    if constexpr (MASKED) {
        const int last_key = CAUSAL ? (qrow < N - 1 ? qrow : N - 1) : N - 1;
        const int ahead = last_key - kv0 - 4 * g;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (32 * b + 8 * (r >> 2) + (r & 3) > ahead) s[b][r] = -INFINITY;
    }
    // ---- online softmax in the log2 domain
    float mx = s[0][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
    mx = pair_max(mx);
    const float tmax = mx * c;
    if (__builtin_amdgcn_ballot_w64(tmax > st.M + kRescaleSlack) != 0) {
        const float Mnew = fmaxf(st.M, tmax);
        const float alpha = (Mnew == -INFINITY) ? 1.0f : fast_exp2(st.M - Mnew);
        st.M = Mnew;
        st.L *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    }
    const float Mref = (MASKED && st.M == -INFINITY) ? 0.f : st.M;
    u4 pf[4];
    const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
    float L = st.L;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = 8 * h + 2 * i;
                const float x0 = fast_exp2(__builtin_fmaf(s[b][r], c, -Mref));
                const float x1 = fast_exp2(__builtin_fmaf(s[b][r + 1], c, -Mref));
                const h2 ph = __builtin_convertvector(f2{x0, x1}, h2);
                // running sum of the rounded probabilities, the values the second product uses
                L = __builtin_amdgcn_fdot2(ph, ones, L, false);
                w[i] = __builtin_bit_cast(unsigned, ph);
            }
            pf[2 * b + h] = w;
        }
    st.L = L;
    // ---- O^T += V_j^T P^T : 4 kv steps x DB row blocks; V^T operands fetched AHEAD steps ahead
    {
        constexpr int NSTEP = 4 * DB, AHEAD = 2;
        auto read_a = [&](int idx) -> s8 {
            const int ks = idx / DB, db = idx % DB;
            const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(ra.v[db][0] + ks * 16 * G::kRowBytes));
            const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(ra.v[db][1] + ks * 16 * G::kRowBytes));
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        };
        s8 av[NSTEP];
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WIDE) mfma_guard(st.o);
#pragma unroll
        for (int idx = 0; idx < AHEAD; ++idx) av[idx] = read_a(idx);
#pragma unroll
        for (int idx = 0; idx < NSTEP; ++idx) {
            if (idx + AHEAD < NSTEP) av[idx + AHEAD] = read_a(idx + AHEAD);
            const int ks = idx / DB, db = idx % DB;
            if constexpr (WIDE) mfma_o(st.o[db], av[idx], pf[ks]);
            else st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, av[idx]), __builtin_bit_cast(h8, pf[ks]),
                                                                   st.o[db], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (WIDE) mfma_settle_a(st.o);
    }
}

// A run of `count` K/V tiles j_first, j_first + step, ... processed one tile at a time (all with or
// all without the mask code).  Self-contained: fetches its first tile itself and leaves with every
// wavefront past the barrier that follows its last tile.  Iteration `it` uses LDS buffer pair it & 1
// and, while computing, fetches the tile of iteration it+1 into the other pair.
template <int D, bool BF16, bool CAUSAL, bool MASKED, int NH>
__device__ __forceinline__ void general_range(TileState<D> (&st)[NH], const LaneMap<D>& lm, const char* Kh, const char* Vh, int N,
                                              float c, int j_first, int step, int count, int qw0, int qrow, int lane,
                                              LDS_PTR(char) lds, bool idle = false) {
    // idle: this wavefront fetches and keeps the barriers like the others but computes nothing (its rows are another
    // wavefront's in this run)
    using G = Geo<D>;
    if (count <= 0) return;
    const unsigned lds0 = (unsigned)(size_t)lds;
    u4 vreg[G::kLoadsPerWave];   // only used for bfloat16 inputs
    // LDS: K buffers at 0 and kTile, V buffers at 2*kTile and 3*kTile.  Start on pair 0.
    ReadAddr<D> ra;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) ra.k[ks] = lds0 + lm.k_rd[ks];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) { ra.v[db][0] = lds0 + 2 * G::kTile + lm.v_rd[db][0]; ra.v[db][1] = lds0 + 2 * G::kTile + lm.v_rd[db][1]; }
    {
        unsigned off[G::kLoadsPerWave];
        tile_offsets<D>(j_first, N, lm, off);
        tile_to_lds<D>(Kh, j_first, off, lm, lds0);
        if constexpr (BF16) {
            tile_to_regs<D>(Vh, j_first, off, vreg);
            regs_to_lds_f16<D>(vreg, lm, lane, lds + 2 * G::kTile);
        } else {
            tile_to_lds<D>(Vh, j_first, off, lm, lds0 + 2 * G::kTile);
        }
        wait_tile_landed();
        __syncthreads();
    }
#pragma unroll 1
    for (int it = 0; it < count; ++it) {
        const int cur = it & 1;
        const int j = j_first + it * step;
        const bool more = it + 1 < count;
        if (more) {
            unsigned off[G::kLoadsPerWave];
            tile_offsets<D>(j + step, N, lm, off);
            tile_to_lds<D>(Kh, j + step, off, lm, lds0 + (cur ^ 1) * G::kTile);
            if constexpr (BF16) tile_to_regs<D>(Vh, j + step, off, vreg);
            else tile_to_lds<D>(Vh, j + step, off, lm, lds0 + (2 + (cur ^ 1)) * G::kTile);
        }
        const int kv0 = j * kTileKV;
#pragma unroll
        for (int h = 0; h < NH; ++h) {   // half h: query rows qw0 + 32h .. +31 (this lane: qrow + 32h)
            const bool active = !idle && qw0 + 32 * h < N && (!CAUSAL || kv0 <= qw0 + 32 * h + 31);
            if (active) compute_tile<D, BF16, CAUSAL, MASKED, NH == 2>(st[h], ra, c, kv0, qrow + 32 * h, lane, N);
        }
        ra.flip(cur ? -G::kTile : G::kTile);
        if (more) {
            if constexpr (BF16) regs_to_lds_f16<D>(vreg, lm, lane, lds + (2 + (cur ^ 1)) * G::kTile);
            wait_tile_landed();
        }
        __syncthreads();
    }
}

// A run of `count` full, unmasked K/V tiles j_first, j_first + step, ..., software pipelined across
// tiles.  While the MFMAs of S(i+1)^T = K(i+1) Q^T run, the exponentials of tile i are issued
// between them; while the MFMAs of O^T += V(i)^T P(i)^T run, the row maximum of S(i+1), the
// lazy-rescale check and the (score*c - M) of tile i+1 are issued between them.  Two register sets
// alternate roles without copies: `A` accumulates the scores of the tile one ahead, `x` holds the
// shifted scores of the current tile until they have become probabilities.  K is therefore fetched
// two tiles ahead and V one tile ahead, still into two LDS buffers each.  For bfloat16 inputs V
// travels global -> registers -> binary16 -> LDS, the conversion spread over the second product.
// Self-contained like general_range().
//
// HALVES: the workgroup walks two runs of `count` tiles at once -- run r = tiles j_first + (r*count + i)*step,
// i = 0..count-1 -- for small problems, where the chip has more compute units than there are query tiles and
// the length of one wavefront's walk is what the launch takes.  All four wavefronts fetch the tiles of both
// runs (a second set of K/V buffers behind the first; for bfloat16 inputs a second set of V registers);
// this wavefront computes on run `run`.
template <int D, bool BF16, bool HALVES = false>
__device__ __forceinline__ void pipelined_range(TileState<D>& st, const LaneMap<D>& lm, const char* Kh, const char* Vh,
                                                float c, int j_first, int step, int count, int lane, LDS_PTR(char) lds,
                                                int run = 0) {
    using G = Geo<D>;
    constexpr int RUNS = HALVES ? 2 : 1;
    constexpr unsigned kSet = 4 * G::kTile;   // one set of buffers: K0 K1 V0 V1
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int NA = 2 * KS;            // MFMAs of one S^T tile
    constexpr int NB = 4 * DB;            // MFMAs of one O^T update
    constexpr int NL = G::kLoadsPerWave;
    constexpr int EU = 16 / NA;           // exp units (2 exp + convert + sum of one pair) per MFMA of phase A
    if (count <= 0) return;
    const unsigned lds0 = (unsigned)(size_t)lds;
    float L_hi = 0.f;   // second partial of the running sum (upper halves of the probability pairs), folded into st.L
    const _Float16 one = opaque_one();
    const f16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f16v A[2];          // S^T of the tile one ahead: block b = keys 32b..32b+31 of the tile
    float x[32];        // score*c - M of the current tile, index 16*b + r
    u4 pf[4];           // its probabilities as B operands
    u4 vreg[(HALVES ? 2 : 1) * NL];   // bfloat16 V chunks in flight (BF16 only), run r in vreg[r * NL ...]

    // LDS read addresses: K of the tile one ahead, V of the current tile
    unsigned rk[KS], rv[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rk[ks] = lds0 + run * kSet + lm.k_rd[ks];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        rv[db][0] = lds0 + run * kSet + 2 * G::kTile + lm.v_rd[db][0];
        rv[db][1] = lds0 + run * kSet + 2 * G::kTile + lm.v_rd[db][1];
    }

    // tile i of run r
    auto tile_base = [&](const char* head, int i, int r = 0) {
        return head + (size_t)(j_first + (r * count + i) * step) * kTileKV * G::kRowBytes;
    };
    auto fetch_burst = [&](const char* head, int i, unsigned dst) {
#pragma unroll
        for (int r = 0; r < RUNS; ++r) {
            const char* base = tile_base(head, i, r);
#pragma unroll
            for (int l = 0; l < NL; ++l) load_to_lds_16B(base, lm.fill_src[l], dst + r * kSet + lm.fill_dst + l * 4096);
        }
    };
    auto k_read = [&](int m) -> u4 { return *(LDS_PTR(u4))(size_t)(rk[m / 2] + (m & 1) * 32 * G::kRowBytes); };
    auto v_read = [&](int idx) -> s8 {
        const int ks = idx / DB, db = idx % DB;
        const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(rv[db][0] + ks * 16 * G::kRowBytes));
        const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(rv[db][1] + ks * 16 * G::kRowBytes));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto rescale = [&](float tmax) {
        st.L += L_hi;
        L_hi = 0.f;
        const float Mnew = fmaxf(st.M, tmax);
        const float alpha = (Mnew == -INFINITY) ? 1.0f : fast_exp2(st.M - Mnew);
        st.M = Mnew;
        st.L *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    };
    float tmax_ahead = 0.f;   // row maximum (times c) of the tile in A, from the latest iteration
    // exp unit u (0..15): the two exponentials of pair u, and the convert + sum of pair u-1
    float e0[16], e1[16];
    auto exp_unit = [&](int u) {
        if (u < 16) {
            e0[u] = fast_exp2(x[2 * u]);
            e1[u] = fast_exp2(x[2 * u + 1]);
        }
        if (u >= 1 && u <= 16) {
            const int v = u - 1;
            const h2 ph = __builtin_convertvector(f2{e0[v], e1[v]}, h2);
            add_pair(st.L, L_hi, ph, one);   // sum of the rounded probabilities, the values the second product uses
            pf[v / 4][v % 4] = __builtin_bit_cast(unsigned, ph);
        }
    };

    // ---------------------------------------------------------------- prologue: tile 0
    fetch_burst(Kh, 0, lds0);
    if constexpr (BF16) {
#pragma unroll
        for (int r = 0; r < RUNS; ++r) {
            const char* base = tile_base(Vh, 0, r);
#pragma unroll
            for (int l = 0; l < NL; ++l) vreg[r * NL + l] = *reinterpret_cast<const u4*>(base + lm.fill_src[l]);
        }
#pragma unroll
        for (int r = 0; r < RUNS; ++r)
#pragma unroll
            for (int l = 0; l < NL; ++l)
                *(LDS_PTR(u4))(lds + r * kSet + 2 * G::kTile + lm.fill_dst + l * 4096 + lane * 16) = bf16x8_to_f16x8(vreg[r * NL + l]);
    } else {
        fetch_burst(Vh, 0, lds0 + 2 * G::kTile);
    }
    wait_tile_landed();
    __syncthreads();
    if (count > 1) fetch_burst(Kh, 1, lds0 + G::kTile);
    {
        u4 a[NA];
        a[0] = k_read(0);
        a[1] = k_read(1);
#pragma unroll
        for (int m = 0; m < NA; ++m) {
            if (m + 2 < NA) a[m + 2] = k_read(m + 2);
            A[m & 1] = mfma_16bit<BF16>(a[m], st.qf[m / 2], m < 2 ? zero : A[m & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        float mx = fmaxf(A[0][0], A[0][1]);
#pragma unroll
        for (int r = 2; r < 32; r += 2) mx = fmaxf(fmaxf(mx, A[r >> 4][r & 15]), A[r >> 4][(r & 15) + 1]);
        const float tmax = pair_max(mx) * c;
        if (__builtin_amdgcn_ballot_w64(!(tmax <= st.M + kRescaleSlack)) != 0) rescale(tmax);
#pragma unroll
        for (int r = 0; r < 32; ++r) x[r] = __builtin_fmaf(A[r >> 4][r & 15], c, -st.M);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rk[ks] += G::kTile;   // K of tile 1 is in buffer 1
    if (count > 1) {
        wait_tile_landed();
        __syncthreads();
    }

    // ---------------------------------------------------------------- steady state: iteration i
    // reads K(i+1) from K buffer (i+1)&1 and V(i) from V buffer i&1; fetches K(i+2) into K buffer
    // i&1 and V(i+1) into V buffer (i+1)&1.  Returns whether the reference maximum has to be raised
    // before tile i+1 can be used.
    auto iteration = [&](int i, auto fetch_k_tag) -> bool {
        constexpr bool FETCH_K = decltype(fetch_k_tag)::value;
        const int cur = i & 1;
        const char* kbase = tile_base(Kh, i + 2);
        const char* vbase = tile_base(Vh, i + 1);
        const char* kbase1 = tile_base(Kh, i + 2, RUNS - 1);   // the same tiles of the second run
        const char* vbase1 = tile_base(Vh, i + 1, RUNS - 1);
        const unsigned kdst = lds0 + cur * G::kTile + lm.fill_dst;
        const unsigned vdst = lds0 + (2 + (cur ^ 1)) * G::kTile + lm.fill_dst;
        // ---- phase A
        {
            u4 a[NA];
            a[0] = k_read(0);
            a[1] = k_read(1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 0; m < NA; ++m) {
                if (m + 2 < NA) a[m + 2] = k_read(m + 2);
                A[m & 1] = mfma_16bit<BF16>(a[m], st.qf[m / 2], m < 2 ? zero : A[m & 1]);
#pragma unroll
                for (int q = 0; q < EU; ++q) exp_unit(m * EU + q);
                // the fetches of an iteration, spread over its first product: K, then V (with two runs: K of
                // both, then V of both, one load per MFMA)
                constexpr int TL = 2 * RUNS * NL;
                if ((m * TL) / NA != ((m + 1) * TL) / NA) {
                    const int li = (m * TL) / NA;
                    const int what = li / NL, l = li % NL;     // what: K run 0, (K run 1,) V run 0, (V run 1)
                    if (what < RUNS) {
                        if (FETCH_K) load_to_lds_16B(what ? kbase1 : kbase, lm.fill_src[l], kdst + what * kSet + l * 4096);
                    } else if constexpr (BF16) {
                        vreg[(what - RUNS) * NL + l] = *reinterpret_cast<const u4*>((what - RUNS ? vbase1 : vbase) + lm.fill_src[l]);
                    } else {
                        load_to_lds_16B(what - RUNS ? vbase1 : vbase, lm.fill_src[l], vdst + (what - RUNS) * kSet + l * 4096);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            exp_unit(16);
        }
        // ---- phase B, first half: row maximum of A and the rescale check
        s8 av[NB];
        av[0] = v_read(0);
        av[1] = v_read(1);
        __builtin_amdgcn_sched_barrier(0);
        float mx = 0.f;
        constexpr int H = NB / 2;          // MFMAs before the check
        constexpr int MS = 2;              // first slot that may read A (MFMA result latency)
        constexpr int MPS = (16 + (H - MS) - 1) / (H - MS);   // max3 ops per slot
#pragma unroll
        for (int idx = 0; idx < H; ++idx) {
            av[idx + 2] = v_read(idx + 2);
            st.o[idx % DB] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, av[idx]), __builtin_bit_cast(h8, pf[idx / DB]),
                                                                    st.o[idx % DB], 0, 0, 0);
            if (idx >= MS) {
#pragma unroll
                for (int q = 0; q < MPS; ++q) {
                    const int op = (idx - MS) * MPS + q;   // op-th max3: elements 2*op, 2*op+1
                    if (op < 16) {
                        const float u0 = A[(2 * op) >> 4][(2 * op) & 15], u1 = A[(2 * op) >> 4][((2 * op) & 15) + 1];
                        mx = op == 0 ? fmaxf(u0, u1) : fmaxf(fmaxf(mx, u0), u1);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        tmax_ahead = pair_max(mx) * c;
        const bool need = __builtin_amdgcn_ballot_w64(!(tmax_ahead <= st.M + kRescaleSlack)) != 0;
        // ---- phase B, second half, with the shifted scores of tile i+1 in between (and, for
        //      bfloat16, the conversion of the fetched V chunks).  If the reference maximum has to
        //      be raised (need), the shifted scores are recomputed after the loop exit.
        constexpr int FPS = 32 / (NB - H);   // fmas per slot
        constexpr int CW = RUNS * NL * 4;                        // 32-bit words of bfloat16 V to convert
        constexpr int CPS = (CW + (NB - H) - 1) / (NB - H);      // ... per slot
#pragma unroll
        for (int idx = H; idx < NB; ++idx) {
            if (idx + 2 < NB) av[idx + 2] = v_read(idx + 2);
            st.o[idx % DB] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, av[idx]), __builtin_bit_cast(h8, pf[idx / DB]),
                                                                    st.o[idx % DB], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < FPS; ++q) {
                const int r = (idx - H) * FPS + q;
                x[r] = __builtin_fmaf(A[r >> 4][r & 15], c, -st.M);
            }
            if constexpr (BF16) {
#pragma unroll
                for (int q = 0; q < CPS; ++q) {
                    const int w = (idx - H) * CPS + q;    // w-th 32-bit word of the fetched chunks
                    if (w < CW) {
                        f2 y;
                        y[0] = __builtin_bit_cast(float, vreg[w / 4][w % 4] << 16);
                        y[1] = __builtin_bit_cast(float, vreg[w / 4][w % 4] & 0xffff0000u);
                        vreg[w / 4][w % 4] = __builtin_bit_cast(unsigned, __builtin_convertvector(y, h2));
                        if (w % 4 == 3)   // chunk w/4 = load (w/4) % NL of run (w/4) / NL
                            *(LDS_PTR(u4))(size_t)(vdst + ((w / 4) / NL) * kSet + ((w / 4) % NL) * 4096 + lane * 16) = vreg[w / 4];
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- switch buffers, publish the fetched tiles
        const int dk = cur ? G::kTile : -G::kTile;   // K(i+2) is in buffer i&1
        const int dv = cur ? -G::kTile : G::kTile;   // V(i+1) is in buffer (i+1)&1
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) rk[ks] += dk;
#pragma unroll
        for (int db = 0; db < DB; ++db) { rv[db][0] += dv; rv[db][1] += dv; }
        wait_tile_landed();
        __syncthreads();
        return need;
    };
    // Raise the reference maximum for the tile held in A and redo its shifted scores; only reached
    // when the loop below stopped because an iteration asked for it.
    auto raise_reference = [&]() {
        rescale(tmax_ahead);
#pragma unroll
        for (int r = 0; r < 32; ++r) x[r] = __builtin_fmaf(A[r >> 4][r & 15], c, -st.M);
    };
    int i = 0;
    while (i + 2 < count) {
        bool need = false;
#pragma unroll 1
        for (; i + 2 < count; ++i) {
            need = iteration(i, std::true_type{});
            if (need) { ++i; break; }
        }
        if (need) raise_reference();
    }
    if (i + 1 < count) {
        const bool need = iteration(i, std::false_type{});
        ++i;
        if (need) raise_reference();
    }

    // ---------------------------------------------------------------- last tile: probabilities, then O^T += V^T P^T
#pragma unroll
    for (int u = 0; u <= 16; ++u) exp_unit(u);
    {
        s8 av[NB];
        av[0] = v_read(0);
        av[1] = v_read(1);
#pragma unroll
        for (int idx = 0; idx < NB; ++idx) {
            if (idx + 2 < NB) av[idx + 2] = v_read(idx + 2);
            st.o[idx % DB] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, av[idx]), __builtin_bit_cast(h8, pf[idx / DB]),
                                                                    st.o[idx % DB], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    st.L += L_hi;
    __syncthreads();   // all reads of the last tile are done before anything refills the buffers
}

// ------------------------------------------------------------------------------------------------
// Wide variant (head dimension 128): a wavefront owns 64 query rows as two 32-row
// halves, a workgroup 256 rows, one workgroup per CU.  Every K and V^T fragment read from LDS feeds
// two MFMAs, one per half, which halves the LDS operand traffic and the L2 -> LDS traffic per flop.
//
// With one wavefront per SIMD the instruction stream of that wavefront is all the SIMD has: an MFMA
// occupies the matrix pipe for 32 cycles, and whatever the wavefront issues between two MFMAs
// (about 5 cycles per vector instruction, 9 per exponential) has to fit under those 32 cycles or the
// pipe idles.  So the vector work per score is cut to the exponential, half a convert, half a
// maximum and the row sum, and spread evenly over the MFMAs:
//   * one FMA per score (score * c - M, c = scale*log2(e) applied to the fp32 score as everywhere else); the
//     row maximum is tracked on the raw scores against the per-row limit (M + slack) / c, so that the test
//     "some score exceeds the slack" costs no multiply;
//   * S^T is computed block by block (kv rows 0..31 of the tile, then 32..63): the exponentials of
//     the second block of tile i run under the first-block MFMAs of S(i+1)^T, which do not touch it,
//     the row sums of tile i under the second-block MFMAs; under the MFMAs of O^T += V(i)^T P(i)^T
//     come the maxima of S(i+1) and the exponentials of its first block, which go into the operand
//     registers of P as the second product releases them.  Those exponentials are taken before the
//     maxima are all known; when a maximum exceeds the slack they are redone (rarely).
// K and V are fetched three and two tiles ahead into four LDS buffers each, so that a fetch has two
// whole iterations to land.
constexpr int kWideBuffers = 4;
constexpr int kWideLdsBytes = 2 * kWideBuffers * Geo<128>::kTile;

template <bool BF16>
__device__ __forceinline__ void pipelined_range_wide(TileState<128> (&st)[2], const LaneMap<128>& lm, const char* Kh,
                                                     const char* Vh, float c, int j_first, int step, int count, int lane,
                                                     LDS_PTR(char) lds) {
    constexpr int D = 128;
    using G = Geo<D>;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int NA = 2 * KS;            // K fragments of one tile (each feeds two MFMAs)
    constexpr int NB = 4 * DB;            // V^T fragments of one tile (each feeds two MFMAs)
    constexpr int NL = G::kLoadsPerWave;
    constexpr unsigned VB = kWideBuffers * G::kTile;   // V buffers follow the K buffers
    constexpr int RA = 2;                 // fragments read ahead where fragments are read one by one (first and last tile)
    if (count <= 0) return;
    const unsigned lds0 = (unsigned)(size_t)lds;
    float L_hi[2] = {0.f, 0.f};   // second partials of the running sums, folded into st[h].L
    const _Float16 one = opaque_one();
    f16v S[2][2];                 // [half][block]: raw scores; pair u = 0..15 of a half is S[h][u / 8][2 * (u % 8) .. + 1]
    float nM[2], lim[2];          // [half]: -M (log2 domain), and the raw score above which M has to be raised
    u4 pf[2][4];                  // [half][contraction step]: probabilities as B operands; pair u is pf[h][u / 4][u % 4]
    float e0[2][16], e1[2][16];
    float tmax_ahead[2] = {0.f, 0.f};   // this lane's maximum of the raw scores of the tile one ahead (never below lim)
    // bfloat16 inputs: K stays bfloat16 (direct loads, bfloat16 MFMAs for S^T); V travels global -> registers ->
    // binary16 -> LDS, because the probabilities are binary16.  vreg holds this wavefront's share of the V tile one
    // ahead between its load (end of an iteration) and its conversion (under the second-block MFMAs of the next).
    u4 vreg[NL];
    const unsigned v_store = lds0 + VB + lm.fill_dst + lane * 16;   // this lane's 16 bytes of load 0 in V buffer 0
    mfma_guard(st[0].o);
    mfma_guard(st[1].o);

    // Tile i of the range lives in K buffer i & 3 and V buffer i & 3.  Fetches beyond the range re-fetch its
    // last tile into a buffer nobody reads, which keeps the loop free of special cases.
    auto tile_base = [&](const char* head, int i) {
        const int ic = i < count ? i : count - 1;
        return head + (size_t)(j_first + ic * step) * kTileKV * G::kRowBytes;
    };
    auto fetch_k = [&](int i, int l) { load_to_lds_16B(tile_base(Kh, i), lm.fill_src[l], lds0 + (i & 3) * G::kTile + lm.fill_dst + l * 4096); };
    auto fetch_v = [&](int i, int l) { load_to_lds_16B(tile_base(Vh, i), lm.fill_src[l], lds0 + VB + (i & 3) * G::kTile + lm.fill_dst + l * 4096); };
    // LDS read addresses of this lane: K of the tile one ahead (buffer 1 at the start), V of the current tile
    unsigned rk[KS], rv[DB][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rk[ks] = lds0 + G::kTile + lm.k_rd[ks];
#pragma unroll
    for (int db = 0; db < DB; ++db) { rv[db][0] = lds0 + VB + lm.v_rd[db][0]; rv[db][1] = lds0 + VB + lm.v_rd[db][1]; }
    // K fragment (ks, b): contraction step ks, kv rows 32b .. 32b+31
    auto k_read = [&](int ks, int b) -> u4 { return *(LDS_PTR(u4))(size_t)(rk[ks] + b * 32 * G::kRowBytes); };
    auto v_read = [&](int idx) -> s8 {
        const int ks = idx / DB, db = idx % DB;
        const s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(rv[db][0] + ks * 16 * G::kRowBytes));
        const s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(size_t)(rv[db][1] + ks * 16 * G::kRowBytes));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // Softmax work items of half h, pair u = 0..15: the two exponentials, the convert into the B operand,
    // the addition to the running sum.
    auto exp2_pair = [&](int h, int u) {
        const float x0 = __builtin_fmaf(S[h][u / 8][2 * (u % 8)], c, nM[h]);
        const float x1 = __builtin_fmaf(S[h][u / 8][2 * (u % 8) + 1], c, nM[h]);
        e0[h][u] = fast_exp2(x0);
        e1[h][u] = fast_exp2(x1);
    };
    auto convert_pair = [&](int h, int u) {
        pf[h][u / 4][u % 4] = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{e0[h][u], e1[h][u]}, h2));
    };
    auto sum_pair = [&](int h, int u) {
        const unsigned word = pf[h][u / 4][u % 4];   // (a copy: bit casts of a vector element do not read that element)
        add_pair(st[h].L, L_hi[h], __builtin_bit_cast(h2, word), one);
    };
    auto first_block_probabilities = [&](int h) {
#pragma unroll
        for (int u = 0; u < 8; ++u) { exp2_pair(h, u); convert_pair(h, u); }
    };
    auto set_reference = [&](int h) {
        nM[h] = -st[h].M;
        // (c is never zero.  The select stays all the same: without it the compiler allocates this kernel's
        // registers differently and spills around the hand-placed MFMAs.)
        lim[h] = c > 0.f ? (st[h].M + kRescaleSlack) / c : INFINITY;
    };

    // ---------------------------------------------------------------- prologue: K(0..2), V(0..1) on their way, S(0)
#pragma unroll
    for (int i = 0; i < 3; ++i) {
#pragma unroll
        for (int l = 0; l < NL; ++l) fetch_k(i, l);
        if constexpr (!BF16) {
            if (i < 2) {
#pragma unroll
                for (int l = 0; l < NL; ++l) fetch_v(i, l);
            }
        }
    }
    if constexpr (BF16) {
        // V(0) goes through registers into buffer 0 now, V(1) waits in vreg for the first iteration
        u4 v0[NL];
#pragma unroll
        for (int l = 0; l < NL; ++l) v0[l] = *reinterpret_cast<const u4*>(tile_base(Vh, 0) + lm.fill_src[l]);
#pragma unroll
        for (int l = 0; l < NL; ++l) vreg[l] = *reinterpret_cast<const u4*>(tile_base(Vh, 1) + lm.fill_src[l]);
#pragma unroll
        for (int l = 0; l < NL; ++l) *(LDS_PTR(u4))(size_t)(v_store + l * 4096) = bf16x8_to_f16x8(v0[l]);
    }
    wait_tile_landed();
    __syncthreads();
    u4 ak[RA];          // the first K fragments of the tile one ahead, read before the iteration starts
    {
        u4 a[NA];       // a[m]: fragment (ks, b) = (m / 2, m % 2) of tile 0 (buffer 0)
        auto k0_read = [&](int m) -> u4 { return *(LDS_PTR(u4))(size_t)(rk[m / 2] - G::kTile + (m & 1) * 32 * G::kRowBytes); };
#pragma unroll
        for (int m = 0; m < RA; ++m) a[m] = k0_read(m);
#pragma unroll
        for (int m = 0; m < NA; ++m) {
            if (m + RA < NA) a[m + RA] = k0_read(m + RA);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (m < 2) mfma_s_first<BF16>(S[h][m & 1], a[m], st[h].qf[m / 2]);
                else mfma_s<BF16>(S[h][m & 1], a[m], st[h].qf[m / 2]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        ak[0] = k_read(0, 0);
        ak[1] = k_read(1, 0);
        mfma_settle_v(S[0][0], S[0][1], S[1][0], S[1][1]);
        mfma_settle_a(st[0].o);
        mfma_settle_a(st[1].o);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float mx = fmaxf(S[h][0][0], S[h][0][1]);
#pragma unroll
            for (int r = 2; r < 32; r += 2) mx = fmaxf(fmaxf(mx, S[h][r >> 4][r & 15]), S[h][r >> 4][(r & 15) + 1]);
            const float tmax = pair_max(mx) * c;
            // the first tile of a query tile finds M = -inf and takes its own maximum as the reference
            if (__builtin_amdgcn_ballot_w64(!(tmax <= st[h].M + kRescaleSlack)) != 0) {
                st[h].L += L_hi[h];
                L_hi[h] = 0.f;
                const float Mnew = fmaxf(st[h].M, tmax);
                const float alpha = (Mnew == -INFINITY) ? 1.0f : fast_exp2(st[h].M - Mnew);
                st[h].M = Mnew;
                st[h].L *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st[h].o[db][r] *= alpha;
            }
            set_reference(h);
            first_block_probabilities(h);
        }
        mfma_guard(st[0].o);
        mfma_guard(st[1].o);
    }

    // ---------------------------------------------------------------- steady state: iteration i
    // enters with the scores of tile i in S and the probabilities of its first block in pf[.][0..1];
    // computes S(i+1)^T from K buffer (i+1)&3 and adds V(i)^T P(i)^T from V buffer i&3; fetches K(i+3) and V(i+2).
    // Its barrier sits in the middle of the second product: by then everything fetched before this
    // iteration (K(i+2), V(i+1) among it) has landed, so the first fragments of the next iteration can be read
    // before this one ends, and the buffers this iteration's fetches overwrite (of K(i-1), V(i-2)) were last
    // read before the previous barrier.  Returns whether a reference maximum has to be raised before
    // tile i+1 can be used.
    auto iteration = [&](int i) -> bool {
        // this iteration's fetches: K(i+3) and V(i+2), source tile bases and LDS destinations of this wavefront
        const char* kbase = tile_base(Kh, i + 3);
        const char* vbase = tile_base(Vh, i + 2);
        const unsigned kdst_s = __builtin_amdgcn_readfirstlane(lds0 + ((i + 3) & 3) * G::kTile + lm.fill_dst);
        const unsigned vdst_s = __builtin_amdgcn_readfirstlane(lds0 + VB + ((i + 2) & 3) * G::kTile + lm.fill_dst);
        s8 av[NB];
        // ---- phase A: S(i+1)^T, block 0 (kv rows 0..31) for both halves, then block 1.
        //      Slot t = 0..31 is the t-th MFMA; fragment n = t / 2 of the block-major order is (ks, b) = (n % 8, n / 8).
        {
            u4 a[NA];   // indexed by n
            a[0] = ak[0];
            a[1] = ak[1];
            // Fragments are read from LDS two at a time, one pair ahead, and used in the order second, first:
            // the one wait for the later read covers both (half as many waits in the instruction stream).
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                if ((q & 1) == 0) {
                    if (q + 2 < NA) { a[q + 2] = k_read((q + 2) % 8, (q + 2) / 8); a[q + 3] = k_read((q + 3) % 8, (q + 3) / 8); }
                    else { av[0] = v_read(0); av[1] = v_read(1); }   // the first V^T fragments of the second product
                }
                const int n = q ^ 1, ks = n % 8, b = n / 8;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int t = 2 * q + h;
                    if (q % 8 == 0) mfma_s_first<BF16>(S[h][b], a[n], st[h].qf[ks]);   // the block's first MFMA
                    else mfma_s<BF16>(S[h][b], a[n], st[h].qf[ks]);
                    if (t < 16) {
                        // exponentials of the second block of tile i: pair 8 + t/2 of half t%2, convert of the one before
                        const int hh = t & 1, u = 8 + t / 2;
                        if (u > 8) convert_pair(hh, u - 1);
                        __builtin_amdgcn_sched_barrier(0);
                        exp2_pair(hh, u);
                    } else {
                        if (t == 16) convert_pair(0, 15);
                        if (t == 17) convert_pair(1, 15);
                        __builtin_amdgcn_sched_barrier(0);
                        // row sums of tile i: words 2(t-16), 2(t-16)+1 of the 32
                        const int w0 = 2 * (t - 16);
                        sum_pair(w0 & 1, w0 >> 1);
                        sum_pair((w0 + 1) & 1, (w0 + 1) >> 1);
                        if constexpr (BF16) {
                            // one word of V(i+1) from bfloat16 to binary16; every fourth completes 16 bytes for LDS
                            const int w = t - 16;
                            const unsigned word = vreg[w / 4][w % 4];
                            f2 y;
                            y[0] = __builtin_bit_cast(float, word << 16);
                            y[1] = __builtin_bit_cast(float, word & 0xffff0000u);
                            vreg[w / 4][w % 4] = __builtin_bit_cast(unsigned, __builtin_convertvector(y, h2));
                            if (w % 4 == 3)
                                *(LDS_PTR(u4))(size_t)(v_store + ((i + 1) & 3) * G::kTile + (w / 4) * 4096) = vreg[w / 4];
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // K read addresses move on to tile i+2
        {
            const int dk = ((i + 2) & 3) ? G::kTile : -3 * G::kTile;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) rk[ks] += dk;
        }
        // ---- phase B: O^T += V(i)^T P(i)^T.  Under its MFMAs (slot t = 0..31): the row maxima of S(i+1) and
        //      their check against the slack (slots 2..9), then the first-block exponentials of tile i+1, whose
        //      converts overwrite pf[.][0] (free after slot 7) and pf[.][1] (free after slot 15).
        float mx[2] = {0.f, 0.f};
        bool need = false;
        auto constexpr_fetch = [&](int li) {
            if (li == 0) load_to_lds_16B_at<0>(kbase, lm.fill_src[0], kdst_s);
            if (li == 1) load_to_lds_16B_at<4096>(kbase, lm.fill_src[1], kdst_s);
            if (li == 2) load_to_lds_16B_at<8192>(kbase, lm.fill_src[2], kdst_s);
            if (li == 3) load_to_lds_16B_at<12288>(kbase, lm.fill_src[3], kdst_s);
            if constexpr (BF16) {
                if (li >= 4) vreg[li - 4] = *reinterpret_cast<const u4*>(vbase + lm.fill_src[li - 4]);
            } else {
                if (li == 4) load_to_lds_16B_at<0>(vbase, lm.fill_src[0], vdst_s);
                if (li == 5) load_to_lds_16B_at<4096>(vbase, lm.fill_src[1], vdst_s);
                if (li == 6) load_to_lds_16B_at<8192>(vbase, lm.fill_src[2], vdst_s);
                if (li == 7) load_to_lds_16B_at<12288>(vbase, lm.fill_src[3], vdst_s);
            }
        };
#pragma unroll
        for (int idx = 0; idx < NB; ++idx) {
            if (idx == NB / 2) {
                // ---- everything fetched before this iteration has landed (all but its own first two loads); publish it
                asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                __syncthreads();
            }
            if ((idx & 1) == 0) {
                if (idx + 2 < NB) { av[idx + 2] = v_read(idx + 2); av[idx + 3] = v_read(idx + 3); }
                else { ak[0] = k_read(0, 0); ak[1] = k_read(1, 0); }   // the first K fragments of the next iteration
            }
            const int f = idx ^ 1;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int t = 2 * idx + h;
                mfma_o(st[h].o[f % DB], av[f], pf[h][f / DB]);
                // the fetches sit in the slots with no other work: two before the barrier, six at the end
                if (t < 2) constexpr_fetch(t);
                if (t >= 26) constexpr_fetch(t - 24);
                if (t >= 2 && t < 10) {
                    // four maxima per slot, the two halves' chains alternating
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = (t - 2) * 4 + q, hh = n & 1, op = n >> 1;    // op-th max3 of half hh
                        const float u0 = S[hh][(2 * op) >> 4][(2 * op) & 15], u1 = S[hh][(2 * op) >> 4][((2 * op) & 15) + 1];
                        mx[hh] = fmaxf(fmaxf(op == 0 ? lim[hh] : mx[hh], u0), u1);   // (starts from lim: exceeds it exactly when a score does)
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (t == 10) {
                    tmax_ahead[0] = mx[0];
                    tmax_ahead[1] = mx[1];
                    need = __builtin_amdgcn_ballot_w64(!(mx[0] <= lim[0]) || !(mx[1] <= lim[1])) != 0;
                }
                if (t >= 10 && t < 18) {            // pairs 0..3 of both halves: pf[.][0]
                    const int hh = t & 1, u = (t - 10) / 2;
                    if (u > 0) convert_pair(hh, u - 1);
                    __builtin_amdgcn_sched_barrier(0);
                    exp2_pair(hh, u);
                }
                if (t >= 18 && t < 26) {            // pairs 4..7: pf[.][1]
                    const int hh = t & 1, u = 4 + (t - 18) / 2;
                    convert_pair(hh, u - 1);
                    __builtin_amdgcn_sched_barrier(0);
                    exp2_pair(hh, u);
                }
                if (t == 26) convert_pair(0, 7);
                if (t == 27) convert_pair(1, 7);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // V read addresses move on to tile i+1
        {
            const int dv = ((i + 1) & 3) ? G::kTile : -3 * G::kTile;
#pragma unroll
            for (int db = 0; db < DB; ++db) { rv[db][0] += dv; rv[db][1] += dv; }
        }
        return need;
    };
    // Between two iterations: the scores of the coming tile exceed the slack somewhere.  The reference maximum
    // of that half goes up (per query row), the sum and the accumulators follow, the scores are taken relative
    // to it and the first-block probabilities are redone.
    auto raise_reference = [&]() {
        mfma_settle_v(S[0][0], S[0][1], S[1][0], S[1][1]);
        mfma_settle_a(st[0].o);
        mfma_settle_a(st[1].o);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // (the comparison is redone on a value the compiler cannot trace back into the loop, or the loop
            // would carry both halves' results along as lane masks)
            float t = tmax_ahead[h];
            asm volatile("" : "+v"(t));
            t = pair_max(t);     // the two lanes of a query row move together
            const bool mine = !(t <= lim[h]);   // (t is the row's maximum only where it exceeds lim)
            if (__builtin_amdgcn_ballot_w64(mine) != 0) {
                const float Mnew = mine ? fmaxf(st[h].M, t * c) : st[h].M;
                const float alpha = fast_exp2(st[h].M - Mnew);
                st[h].M = Mnew;
                st[h].L = (st[h].L + L_hi[h]) * alpha;
                L_hi[h] = 0.f;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st[h].o[db][r] *= alpha;
                set_reference(h);
                first_block_probabilities(h);
            }
        }
        mfma_guard(st[0].o);
        mfma_guard(st[1].o);
    };
    int i = 0;
    while (i + 1 < count) {
        bool need = false;
#pragma unroll 1
        for (; i + 1 < count; ++i) {
            need = iteration(i);
            if (need) { ++i; break; }
        }
        if (need) raise_reference();
    }

    // ---------------------------------------------------------------- last tile: the rest of its probabilities, then O^T += V^T P^T
    mfma_settle_v(S[0][0], S[0][1], S[1][0], S[1][1]);
#pragma unroll
    for (int u = 8; u < 16; ++u) {
#pragma unroll
        for (int h = 0; h < 2; ++h) { exp2_pair(h, u); convert_pair(h, u); }
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) { sum_pair(0, u); sum_pair(1, u); }
    {
        s8 av[NB];
#pragma unroll
        for (int idx = 0; idx < RA; ++idx) av[idx] = v_read(idx);
#pragma unroll
        for (int idx = 0; idx < NB; ++idx) {
            if (idx + RA < NB) av[idx + RA] = v_read(idx + RA);
#pragma unroll
            for (int h = 0; h < 2; ++h) mfma_o(st[h].o[idx % DB], av[idx], pf[h][idx / DB]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    st[0].L += L_hi[0];
    st[1].L += L_hi[1];
    mfma_settle_a(st[0].o);   // the accumulators are complete before the caller's vector code reads them
    mfma_settle_a(st[1].o);
    wait_tile_landed();   // also the fetches past the end of the range
    __syncthreads();      // all reads of the last tile are done before anything refills the buffers
}

// The epilogue where variant.qo_streaming asks for it: O leaves through LDS so that a store instruction writes whole
// 128-byte lines (8 rows x 128 bytes per instruction, 16 bytes per lane), marked non-temporal: the rows of O are written
// once and never read by the kernel, and written this way they do not take the place of K/V tiles in the L2.
// (Non-temporal stores of the 8- and 16-byte pieces a lane holds per row are not gathered into lines by the L2 and cost
// several times the write traffic.)  `stage` is 4 KiB of LDS of this wavefront's own: 32 rows x 128 bytes, the 16-byte
// chunk c of row r at chunk position c ^ (r & 7), filled by the caller with one 128-byte column block of its 32 rows.
// drain_stage() writes that block out: `dst` points at the block's first row in O, row_bytes is O's row pitch,
// rows_left the number of the 32 rows that lie inside the sequence (<= 0: none).
__device__ __forceinline__ void stage_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }
__device__ __forceinline__ void drain_stage(LDS_PTR(char) stage, char* dst, size_t row_bytes, int rows_left, int lane) {
    stage_fence();
    const int chunk = lane & 7;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = 8 * k + (lane >> 3);
        const u4 x = *(LDS_PTR(u4))(stage + row * 128 + ((chunk ^ (row & 7)) << 4));
        char* to = dst + row * row_bytes + chunk * 16;
        // (the s_nop: a store of more than 8 bytes reads its data registers up to two cycles after issue, and the compiler
        //  does not see a store in this statement when it decides what may overwrite them next)
        if (row < rows_left) asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 1" ::"v"(to), "v"(x) : "memory");
    }
    stage_fence();
}

// One query tile (Alg. 1 body): rows [t*128*NH, (t+1)*128*NH) of head `hh`, K/V tiles j0, j0+step, ... (nkv of
// them).  A wavefront owns NH halves of 32 query rows each (NH = 2: the wide variant).
// HALVES (32 rows per wavefront): the tile has 64 rows; of its full, unmasked K/V tiles wavefronts
// 0 and 1 take the first half and wavefronts 2 and 3, for the same rows, the second half, at once, and the two partial
// results are merged through LDS (the merge of two softmax partials: common reference maximum, both rescaled to it).
// What does not split evenly or needs the mask -- an odd plain tile, the diagonal tile, a ragged last tile -- is taken
// one tile at a time by wavefronts 0 and 1 alone, after the merge in a forward scan and before the halves in a
// backward one, where it comes first.
template <int D, bool BF16, bool CAUSAL, int NH, bool HALVES = false>
__device__ __forceinline__ void process_q_tile(const Params& p, const LaneMap<D>& lm, int hh, int t, int j0, int step,
                                               int nkv, int wave, int lane, LDS_PTR(char) lds) {
    static_assert(!HALVES || NH == 1, "two key ranges at once: 32-row kernel");
    using G = Geo<D>;
    constexpr int KS = D / 16;    // MFMA steps along d for S^T
    constexpr int DB = D / 32;    // 32-row blocks of O^T
    constexpr int TQ = HALVES ? kTileQ / 2 : kTileQ * NH;
    const int g = lane >> 5, ln = lane & 31;
    const int N = p.N;
    const size_t head_off = (size_t)hh * N * G::kRowBytes;
    const char* Qh = static_cast<const char*>(p.Q) + head_off;
    const char* Kh = static_cast<const char*>(p.K) + head_off;
    const char* Vh = static_cast<const char*>(p.V) + head_off;

    const int run = HALVES ? wave >> 1 : 0;                            // which half of the scan this wavefront computes
    const int qw0 = t * TQ + (HALVES ? wave & 1 : wave) * 32 * NH;     // first query row of this wavefront
    const int qrow = qw0 + ln;                // this lane's query row in half 0 (column of S^T)

    TileState<D> st[NH];
    // With variant.qo_streaming the rows of Q come in the way K tiles do -- 64 rows at a time straight into LDS, whole
    // lines per instruction, the four wavefronts together -- but marked non-temporal, and are read from there in the
    // K operand's pattern, which is also Q's.  The buffers are free: the last range of the previous tile ended with a barrier.
    unsigned q_at = 0;     // byte offset in LDS of this lane's first fragment of half 0
    if (p.stream_q) {
        int l2 = lane;
        asm volatile("" : "+v"(l2));        // (a lane map of its own that does not live on: see the note on registers below)
        const LaneMap<D> lq(wave, l2);
        const unsigned lds0 = (unsigned)(size_t)lds;
#pragma unroll
        for (int m = 0; m < TQ / kTileKV; ++m) {
            const int q0 = t * TQ + m * kTileKV;
            const int first = q0 < N ? q0 : N - 1;          // rows beyond N repeat row N-1, as below
            const char* base = Qh + (size_t)first * G::kRowBytes;
#pragma unroll
            for (int i = 0; i < G::kLoadsPerWave; ++i) {
                const int row = lq.fill_src[i] / G::kRowBytes, chunk = lq.fill_src[i] % G::kRowBytes;
                const int r = q0 + row < N ? q0 + row : N - 1;
                load_to_lds_16B_nt(base, (unsigned)((r - first) * G::kRowBytes + chunk), lds0 + m * G::kTile + lq.fill_dst + i * 4096);
            }
        }
        const int mine = HALVES ? wave & 1 : wave;           // which 32 * NH rows of the tile are this wavefront's
        q_at = (mine * NH / 2) * G::kTile + ((mine * NH) & 1) * 32 * G::kRowBytes + lq.k_rd[0];
        wait_tile_landed();
        __syncthreads();
    }
    int lane_q = lane;
    asm volatile("" : "+v"(lane_q));      // (addresses used once: built from a copy of the lane index of their own)
#pragma unroll
    for (int h = 0; h < NH; ++h) {   // rows beyond N repeat row N-1 (computed, never stored)
        const int qr = qw0 + (lane_q & 31) + 32 * h < N ? qw0 + (lane_q & 31) + 32 * h : N - 1;
        const char* qp = Qh + (size_t)qr * G::kRowBytes + (lane_q >> 5) * 16;
        const unsigned flip = p.negate_q ? 0x80008000u : 0u;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            // (chunk 2 ks + g of a row sits at chunk position (2 ks + g) ^ swz(row): k_rd[ks] = k_rd[0] ^ (32 ks))
            u4 v = p.stream_q ? *(LDS_PTR(u4))(lds + ((q_at + h * 32 * G::kRowBytes) ^ (unsigned)(ks * 32)))
                              : *reinterpret_cast<const u4*>(qp + ks * 32);
            v[0] ^= flip; v[1] ^= flip; v[2] ^= flip; v[3] ^= flip;
            if constexpr (NH == 2) {
                if constexpr (!BF16) {
                    if (p.q_bf16) v = bf16x8_to_f16x8(v);   // K and V are binary16 copies: Q follows (exact for normal binary16 magnitudes)
                }
                asm volatile("" : "=a"(st[h].qf[ks]) : "0"(v));   // accumulation registers from here on
            } else {
                st[h].qf[ks] = v;
            }
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[h].o[db][r] = 0.f;
        st[h].M = -INFINITY;
        st[h].L = 0.f;
    }
    if (p.stream_q) __syncthreads();      // the fragments are in registers before the first K/V fetch overwrites the rows
    const float c = p.c;

    // Tiles with index >= jm need the mask code: the ragged last tile, and under the causal mask
    // the tiles that reach past the first row of this query tile.  They sit at one end of the scan,
    // so the scan is a pipelined run of plain tiles and a run of masked tiles, in scan order.
    const int kv_tiles = (N + kTileKV - 1) / kTileKV;
    const int jm = CAUSAL ? (t * TQ) / kTileKV : ((N % kTileKV) ? kv_tiles - 1 : kv_tiles);
    const int n_masked = nkv > jm ? nkv - jm : 0;
    const int n_plain = nkv - n_masked;
    // (The wide variant has no registers to spare: each of its runs builds the per-lane address tables afresh,
    // from a lane index the compiler cannot see through, so that none of them stays live across the other run.)
    auto plain = [&](int j_first) {
        if constexpr (NH == 1) {
            pipelined_range<D, BF16>(st[0], lm, Kh, Vh, c, j_first, step, n_plain, lane, lds);
        } else {
            int l2 = lane;
            asm volatile("" : "+v"(l2));
            const LaneMap<D> lm2(wave, l2);
            pipelined_range_wide<BF16>(st, lm2, Kh, Vh, c, j_first, step, n_plain, l2, lds);
        }
    };
    auto masked = [&](int j_first) {
        if constexpr (NH == 1) {
            general_range<D, BF16, CAUSAL, true, NH>(st, lm, Kh, Vh, N, c, j_first, step, n_masked, qw0, qrow, lane, lds);
        } else {
            int l2 = lane;
            asm volatile("" : "+v"(l2));
            const LaneMap<D> lm2(wave, l2);
            general_range<D, BF16, CAUSAL, true, NH>(st, lm2, Kh, Vh, N, c, j_first, step, n_masked, qw0, qrow, l2, lds);
        }
    };
    if constexpr (HALVES) {
        const int half = n_plain / 2;                       // plain tiles per run
        const int n_left = (n_plain & 1) + n_masked;        // tiles left for the tile-at-a-time code
        if (step < 0)
            general_range<D, BF16, CAUSAL, true, NH>(st, lm, Kh, Vh, N, c, j0, step, n_left, qw0, qrow, lane, lds, run == 1);
        pipelined_range<D, BF16, true>(st[0], lm, Kh, Vh, c, step > 0 ? j0 : j0 + n_left * step, step, half, lane, lds, run);
        // ---- merge: wavefront w + 2 hands (O^T, M, L) of its half to wavefront w, lane to lane, through LDS
        //      (value k of lane l of wavefront w + 2 at float index (2k + w) * 64 + l: no bank conflicts)
        constexpr int NV = DB * 16 + 2;
        LDS_PTR(float) xch = (LDS_PTR(float))lds;
        if (run == 1) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[(2 * (db * 16 + r) + (wave & 1)) * 64 + lane] = st[0].o[db][r];
            xch[(2 * (NV - 2) + (wave & 1)) * 64 + lane] = st[0].M;
            xch[(2 * (NV - 1) + (wave & 1)) * 64 + lane] = st[0].L;
        }
        __syncthreads();
        if (run == 0) {
            const float M1 = xch[(2 * (NV - 2) + wave) * 64 + lane], L1 = xch[(2 * (NV - 1) + wave) * 64 + lane];
            const float M = fmaxf(st[0].M, M1);
            const float a0 = st[0].M == -INFINITY ? 0.f : fast_exp2(st[0].M - M);
            const float a1 = M1 == -INFINITY ? 0.f : fast_exp2(M1 - M);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    st[0].o[db][r] = st[0].o[db][r] * a0 + xch[(2 * (db * 16 + r) + wave) * 64 + lane] * a1;
            st[0].M = M;
            st[0].L = st[0].L * a0 + L1 * a1;
        }
        __syncthreads();   // the exchange area is read before the next fetches overwrite it
        if (step > 0)
            general_range<D, BF16, CAUSAL, true, NH>(st, lm, Kh, Vh, N, c, j0 + 2 * half * step, step, n_left, qw0, qrow, lane,
                                                     lds, run == 1);
    } else if (step > 0) {
        plain(j0);
        masked(j0 + n_plain * step);
    } else {
        masked(j0);
        plain(j0 + n_masked * step);
    }

    // ---- epilogue: O_i = acc / l  (the division Alg. 1 leaves implicit; Eq. 1 fixes it)
    const bool writes = !HALVES || run == 0;     // of two wavefronts that share rows, the first holds the merged result
    const int lane_in = lane;
    if (p.stream_o) {
        wait_tile_landed();
        __syncthreads();          // nothing is on its way into the K/V buffers any more: they serve as staging area
        if (writes) {
            LDS_PTR(char) stage = lds + wave * 4096;
            int lane = lane_in;
            asm volatile("" : "+v"(lane));     // lane-derived addresses are built here, not carried across the scan
            const int g = lane >> 5, ln = lane & 31;
            const int sw = ln & 7;
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float inv = 1.0f / pair_sum(st[h].L);
                const int row0 = qw0 + 32 * h;
                const int rows_left = N - row0;      // <= 0: the whole half lies beyond the sequence
                if (p.o_dtype == SAWATTN_F32) {
                    constexpr size_t RB = (size_t)D * 4;
                    char* dst = static_cast<char*>(p.O) + ((size_t)hh * N + row0) * RB;
#pragma unroll
                    for (int db = 0; db < DB; ++db) {          // 32 columns = 128 bytes per row
                        const f16v& o = st[h].o[db];
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const f4 v = {o[4 * rq] * inv, o[4 * rq + 1] * inv, o[4 * rq + 2] * inv, o[4 * rq + 3] * inv};
                            *(LDS_PTR(f4))(stage + ln * 128 + (((2 * rq + g) ^ sw) << 4)) = v;
                        }
                        drain_stage(stage, dst + db * 128, RB, rows_left, lane);
                    }
                } else {
                    constexpr size_t RB = (size_t)D * 2;
                    char* dst = static_cast<char*>(p.O) + ((size_t)hh * N + row0) * RB;
#pragma unroll
                    for (int pass = 0; pass < DB / 2; ++pass) {   // 64 columns = 128 bytes per row
#pragma unroll
                        for (int dbl = 0; dbl < 2; ++dbl) {
                            const f16v& o = st[h].o[2 * pass + dbl];
#pragma unroll
                            for (int rq = 0; rq < 4; ++rq) {
                                const f4 v = {o[4 * rq] * inv, o[4 * rq + 1] * inv, o[4 * rq + 2] * inv, o[4 * rq + 3] * inv};
                                LDS_PTR(char) at = stage + ln * 128 + (((4 * dbl + rq) ^ sw) << 4) + 8 * g;
                                if (p.o_dtype == SAWATTN_F16) *(LDS_PTR(h4))at = __builtin_convertvector(v, h4);
                                else *(LDS_PTR(b4))at = __builtin_convertvector(v, b4);
                            }
                        }
                        drain_stage(stage, dst + pass * 128, RB, rows_left, lane);
                    }
                }
            }
        }
        __syncthreads();          // the staging area is read before the next tile's fetches overwrite it
        return;
    }
    if (!writes) return;
    int lane_out = lane_in;
    asm volatile("" : "+v"(lane_out));
    const int g_out = lane_out >> 5, qrow_out = qw0 + (lane_out & 31);
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const float inv = 1.0f / pair_sum(st[h].L);
        if (qrow_out + 32 * h < N) {
            const size_t orow = ((size_t)hh * N + qrow_out + 32 * h) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const f16v& o = st[h].o[db];
                    f4 v = {o[4 * rq] * inv, o[4 * rq + 1] * inv, o[4 * rq + 2] * inv, o[4 * rq + 3] * inv};
                    const size_t col = 32 * db + 8 * rq + 4 * g_out;
                    if (p.o_dtype == SAWATTN_F32) {
                        *reinterpret_cast<f4*>(static_cast<float*>(p.O) + orow + col) = v;
                    } else if (p.o_dtype == SAWATTN_F16) {
                        *reinterpret_cast<h4*>(static_cast<_Float16*>(p.O) + orow + col) = __builtin_convertvector(v, h4);
                    } else {
                        *reinterpret_cast<b4*>(static_cast<__bf16*>(p.O) + orow + col) = __builtin_convertvector(v, b4);
                    }
                }
        }
    }
}

// bfloat16 -> binary16 copies of K and V for the workspace path (16 bytes per lane and step).
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(const u4* __restrict__ K, const u4* __restrict__ V,
                                                          u4* __restrict__ K16, u4* __restrict__ V16, size_t chunks) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += stride) {
        K16[i] = bf16x8_to_f16x8(K[i]);
        V16[i] = bf16x8_to_f16x8(V[i]);
    }
}

// Re-alignment of the workgroups of one cache domain.  The reuse the schedule is built on (Sec. 3.4)
// needs the workgroups that share an L2 to walk the same K/V at about the same time.  They start
// aligned and do the same number of tile steps per head, but nothing keeps them aligned: measured
// over 16 heads per domain their drift grows past what the L2 holds and the hit rate falls from
// 95 % to 55 %.  So between two heads the workgroups of a domain wait for each other on a ticket
// counter.  The wait is bounded: if the workgroups are not all resident (a shared GPU), it gives
// up after kSyncSpinLimit polls and the kernel carries on unaligned; results never depend on it.
// The counters are library-owned device memory: kTicketSets sets of one counter per domain.  Every
// launch that uses them takes the next set in turn (a host-side count) and clears it with a
// one-wavefront kernel enqueued just before it, so launches that overlap on one GPU -- other streams,
// other host threads -- do not disturb each other unless kTicketSets or more of them are in flight;
// then they may lose the alignment and wait out the bound (about 8 ms per head boundary at worst),
// never more.
constexpr int kTicketSets = 8;
__device__ unsigned g_domain_tickets[kTicketSets][kDomains];
constexpr int kSyncSpinLimit = 1 << 14;     // polls of about 1000 cycles each

__global__ void clear_tickets_kernel(int set) {
    if (threadIdx.x < kDomains) g_domain_tickets[set][threadIdx.x] = 0u;
}

// Called by every workgroup of `domain` the same number of times; `slots` workgroups take part.
__device__ __forceinline__ void domain_sync(int set, int domain, int slots) {
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned* t = &g_domain_tickets[set][domain];
        const unsigned mine = __hip_atomic_fetch_add(t, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned target = (mine / (unsigned)slots + 1u) * (unsigned)slots;
        for (int spin = 0; spin < kSyncSpinLimit; ++spin) {
            if ((int)(__hip_atomic_load(t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0) break;
            __builtin_amdgcn_s_sleep(16);
        }
    }
    __syncthreads();
}

template <int D, bool BF16, bool CAUSAL, int NH, bool HALVES = false>
__global__ __launch_bounds__(kThreads, HALVES ? (D == 64 ? 2 : 1) : NH == 2 ? 1 : (D == 64 ? 3 : 2)) void attn_fwd_kernel(Params p) {
    extern __shared__ __align__(16) char smem[];
    const Schedule& s = p.sched;
    const int lane0 = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int local = 0;           // query tiles this workgroup has processed
    for (int it = 0; it < s.local_iters; ++it) {
        const Work w = decode_work(s, (int)blockIdx.x, it, CAUSAL, p.sawtooth != 0);
        if (w.tile >= 0) {
            const int nkv = visible_kv_tiles(s, w.tile, p.N, CAUSAL);
            const int j0 = w.backward ? nkv - 1 : 0;
            const int step = w.backward ? -1 : 1;
            if (p.trace && threadIdx.x == 0) {
                int32_t* rec = p.trace + ((size_t)blockIdx.x * p.max_local + local) * 4;
                rec[0] = w.head; rec[1] = w.tile; rec[2] = j0; rec[3] = j0 + (nkv - 1) * step;
            }
            // The per-lane address tables are rebuilt for every query tile from a lane index the
            // compiler cannot see through, so that they are not kept in registers across the loops.
            int lane = lane0;
            asm volatile("" : "+v"(lane));
            const LaneMap<D> lm(wave, lane);
            process_q_tile<D, BF16, CAUSAL, NH, HALVES>(p, lm, w.head, w.tile, j0, step, nkv, wave, lane, (LDS_PTR(char))smem);
            ++local;
        }
        // Every workgroup of the domain comes here once per head, also those that sat rounds out.
        // (With the align_rounds variant also once per round: measured, it changes neither the L2 traffic
        // nor the time of the kernel with 64 rows per wavefront, whose workgroups stay in step by themselves.)
        if (w.sync_after) domain_sync(p.ticket_set, (int)blockIdx.x % kDomains, s.slots);
    }
    if (p.trace_count && threadIdx.x == 0) p.trace_count[blockIdx.x] = local;
}


// ------------------------------------------------------------------------------------------- host

thread_local char g_err[256] = "";

int fail(int code, const char* msg) {
    std::snprintf(g_err, sizeof g_err, "%s", msg);
    return code;
}

int check_shape(int B, int H, int N, int d) {
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return fail(SAWATTN_ERR_INVALID_ARG, "B, H, N and d must be positive");
    if (d != 64 && d != 128) return fail(SAWATTN_ERR_UNSUPPORTED, "head dimension must be 64 or 128");
    const long long heads = (long long)B * H;
    if (heads >= (1LL << 31) / kDomains) return fail(SAWATTN_ERR_INVALID_ARG, "B*H too large");
    const long long q_tiles = (N + (long long)kTileQ - 1) / kTileQ;
    if (heads * q_tiles >= (1LL << 31)) return fail(SAWATTN_ERR_INVALID_ARG, "B*H*ceil(N/128) must be below 2^31");
    if ((double)heads * (double)N * (double)d >= 1099511627776.0) return fail(SAWATTN_ERR_INVALID_ARG, "B*H*N*d must be below 2^40");
    return SAWATTN_OK;
}

void fill_info(const Schedule& s, int d, sawattn_launch_info* out) {
    out->tile_q = s.tile_q;
    out->tile_kv = kTileKV;
    out->block_threads = kThreads;
    out->grid = s.grid;
    out->lds_bytes = s.tile_q > kTileQ ? kWideLdsBytes
                                       : (s.tile_q < kTileQ ? 2 : 1) * (d == 128 ? Geo<128>::kLdsBytes : Geo<64>::kLdsBytes);
    out->domains = kDomains;
    out->slots = s.slots;
    out->parts_per_head = s.parts;
    out->q_tiles_per_head = s.q_tiles;
    out->max_local_tiles = s.local_iters;
    out->launch = s.launch == kLaunchGrid ? SAWATTN_LAUNCH_GRID : SAWATTN_LAUNCH_PERSISTENT;
    out->tiles_per_workgroup = s.tiles_per_wg;
    out->qo_streaming = s.qo_streaming;
}

std::atomic<unsigned> g_ticket_turn{0};

template <int D, bool BF16, bool CAUSAL, int NH, bool HALVES = false>
int launch(Params& p, int grid, hipStream_t stream) {
    auto kern = attn_fwd_kernel<D, BF16, CAUSAL, NH, HALVES>;
    constexpr int lds_bytes = NH == 2 ? kWideLdsBytes : (HALVES ? 2 : 1) * Geo<D>::kLdsBytes;
    // The LDS size a kernel may ask for is a per-device attribute of the function: set once per device (bit = device).
    static std::atomic<unsigned long long> configured{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return fail(SAWATTN_ERR_RUNTIME, "hipGetDevice failed (or more than 64 devices)");
    }
    if (!(configured.load(std::memory_order_acquire) >> dev & 1ull)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                lds_bytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(SAWATTN_ERR_RUNTIME, "hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed");
        }
        configured.fetch_or(1ull << dev, std::memory_order_release);
    }
    p.ticket_set = 0;
    if (p.sched.sync_heads || p.sched.sync_rounds) {
        p.ticket_set = (int)(g_ticket_turn.fetch_add(1u, std::memory_order_relaxed) % (unsigned)kTicketSets);
        hipLaunchKernelGGL(clear_tickets_kernel, dim3(1), dim3(64), 0, stream, p.ticket_set);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds_bytes, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        char msg[200];
        std::snprintf(msg, sizeof msg, "kernel launch failed: %s", hipGetErrorString(e));
        return fail(SAWATTN_ERR_RUNTIME, msg);
    }
    return SAWATTN_OK;
}

// Validates a variant description (NULL = the default schedule) and builds its schedule.
int schedule_for(int B, int H, int N, int d, bool causal, bool bf16, const sawattn_variant* v, Schedule* out) {
    int launch = -1 /* chosen below */, decode = kDecodeDomain, max_slots = 0, tiles_per_wg = 0, rows = 0, halves = 0;
    bool align_rounds = false;
    if (v) {
        if (v->kv_halves < 0 || v->kv_halves > 2)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.kv_halves must be 0 (default), 1 or 2");
        halves = v->kv_halves;
        if (halves == 2) {
            if (v->rows_per_wavefront == 64)
                return fail(SAWATTN_ERR_UNSUPPORTED, "variant.kv_halves = 2 goes with 32 rows per wavefront");
        }
        if (v->launch != SAWATTN_LAUNCH_PERSISTENT && v->launch != SAWATTN_LAUNCH_GRID && v->launch != SAWATTN_LAUNCH_AUTO)
            return fail(SAWATTN_ERR_INVALID_ARG,
                        "variant.launch must be SAWATTN_LAUNCH_PERSISTENT, SAWATTN_LAUNCH_GRID or SAWATTN_LAUNCH_AUTO");
        if (v->decode != SAWATTN_DECODE_DOMAIN && v->decode != SAWATTN_DECODE_LINEAR)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.decode must be SAWATTN_DECODE_DOMAIN or SAWATTN_DECODE_LINEAR");
        if (v->rows_per_wavefront != 0 && v->rows_per_wavefront != 32 && v->rows_per_wavefront != 64)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.rows_per_wavefront must be 0 (default), 32 or 64");
        if (v->rows_per_wavefront == 64 && d != 128)
            return fail(SAWATTN_ERR_UNSUPPORTED, "variant.rows_per_wavefront = 64 needs head dimension 128");
        rows = v->rows_per_wavefront;
        if (halves == 0) halves = rows == 64 ? 1 : default_kv_halves(B * H, N, d, causal, bf16);
        if (halves == 2) rows = 32;
        if (rows == 0) rows = v->slots_per_domain > resident_slots(d, 2 * kTileQ) ? 32 : default_rows_per_wavefront(B * H, N, d, causal, bf16);
        if (v->slots_per_domain < 0 ||
            v->slots_per_domain > resident_slots(d, rows == 64 ? 2 * kTileQ : (halves == 2 ? kTileQ / 2 : kTileQ)))
            return fail(SAWATTN_ERR_INVALID_ARG,
                        "variant.slots_per_domain must be 0 (default) or 1..64 (1..96 for d = 64, 1..32 with 64 rows per "
                        "wavefront; with kv_halves = 2: 1..64 for d = 64, 1..32 for d = 128)");
        if (v->tiles_per_workgroup < 0 || v->tiles_per_workgroup > 2)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.tiles_per_workgroup must be 0 (default), 1 or 2");
        if (v->launch != SAWATTN_LAUNCH_AUTO) launch = v->launch == SAWATTN_LAUNCH_GRID ? kLaunchGrid : kLaunchPersistent;
        decode = v->decode == SAWATTN_DECODE_LINEAR ? kDecodeLinear : kDecodeDomain;
        max_slots = v->slots_per_domain;
        if (v->tiles_per_workgroup) tiles_per_wg = v->tiles_per_workgroup;
        if (v->qo_streaming < 0 || v->qo_streaming > 4)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.qo_streaming must be 0 (default), 1 (O), 2 (Q), 3 (both) or 4 (neither)");
        if (v->align_rounds != 0 && v->align_rounds != 1)
            return fail(SAWATTN_ERR_INVALID_ARG, "variant.align_rounds must be 0 or 1");
        align_rounds = v->align_rounds == 1;
    }
    if (halves == 0) halves = default_kv_halves(B * H, N, d, causal, bf16);
    if (halves == 2) rows = 32;
    if (rows == 0) rows = default_rows_per_wavefront(B * H, N, d, causal, bf16);
    const int tile_q = rows == 64 ? 2 * kTileQ : (halves == 2 ? kTileQ / 2 : kTileQ);
    if (launch < 0) {
        // the caller leaves the launch open: persistent, or for short heads the direct launch with one tile each
        launch = decode == kDecodeDomain && max_slots == 0 ? default_launch(B * H, N, d, causal, tile_q) : kLaunchPersistent;
        if (launch == kLaunchGrid && tiles_per_wg == 0) tiles_per_wg = 1;
    }
    if (tiles_per_wg == 0) tiles_per_wg = 2;
    if (max_slots == 0) max_slots = resident_slots(d, tile_q);
    *out = make_schedule(B * H, N, causal, launch, decode, max_slots, tiles_per_wg, tile_q, align_rounds);
    out->qo_streaming = v && v->qo_streaming ? v->qo_streaming : default_qo_streaming(N, d);
    return SAWATTN_OK;
}

// Whether bfloat16 inputs, converted to binary16, would run the wide variant: then a workspace pays.
int workspace_schedule(int B, int H, int N, int d, bool causal, bool bf16, const sawattn_variant* v, Schedule* out,
                       bool* use) {
    *use = false;
    if (!bf16 || d != 128) return SAWATTN_OK;
    Schedule s;
    const int rc = schedule_for(B, H, N, d, causal, false, v, &s);
    if (rc != SAWATTN_OK) return rc;
    if (s.tile_q > kTileQ) { *use = true; *out = s; }
    return SAWATTN_OK;
}

int run(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale, int causal,
        int scan_order, int in_dtype, int o_dtype, void* hip_stream, const sawattn_variant* variant, int32_t* trace,
        int32_t* trace_count, void* workspace = nullptr, size_t workspace_bytes = 0) {
    int rc = check_shape(B, H, N, d);
    if (rc != SAWATTN_OK) return rc;
    if (!Q || !K || !V || !O) return fail(SAWATTN_ERR_INVALID_ARG, "Q, K, V and O must be non-null");
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15u)
        return fail(SAWATTN_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    if (!std::isfinite(scale)) return fail(SAWATTN_ERR_INVALID_ARG, "scale must be finite");
    if (scan_order != SAWATTN_SCAN_CYCLIC && scan_order != SAWATTN_SCAN_SAWTOOTH)
        return fail(SAWATTN_ERR_INVALID_ARG, "scan_order must be SAWATTN_SCAN_CYCLIC or SAWATTN_SCAN_SAWTOOTH");
    if (in_dtype != SAWATTN_F16 && in_dtype != SAWATTN_BF16)
        return fail(SAWATTN_ERR_INVALID_ARG, "in_dtype must be SAWATTN_F16 or SAWATTN_BF16");
    if (o_dtype != SAWATTN_F16 && o_dtype != SAWATTN_BF16 && o_dtype != SAWATTN_F32)
        return fail(SAWATTN_ERR_INVALID_ARG, "o_dtype must be SAWATTN_F16, SAWATTN_BF16 or SAWATTN_F32");
    if ((trace == nullptr) != (trace_count == nullptr))
        return fail(SAWATTN_ERR_INVALID_ARG, "trace and trace_count must be given together");
    Schedule sched;
    bool converted = false;   // bfloat16 inputs through binary16 copies of K and V in the caller's workspace
    if (workspace) {
        rc = workspace_schedule(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &sched, &converted);
        if (rc != SAWATTN_OK) return rc;
    }
    if (!converted) {
        rc = schedule_for(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &sched);
        if (rc != SAWATTN_OK) return rc;
    }
    {   // A workgroup writes its O rows while others still read Q, K, V: O may not share memory with them.
        const unsigned long long elems = (unsigned long long)B * H * N * d;
        const unsigned long long in_bytes = elems * 2u, out_bytes = elems * (o_dtype == SAWATTN_F32 ? 4u : 2u);
        const uintptr_t o0 = (uintptr_t)O, o1 = o0 + out_bytes;
        for (const void* in : {Q, K, V}) {
            const uintptr_t i0 = (uintptr_t)in, i1 = i0 + in_bytes;
            if (o0 < i1 && i0 < o1) return fail(SAWATTN_ERR_INVALID_ARG, "O must not overlap Q, K or V");
        }
        if (converted) {
            if ((uintptr_t)workspace & 15u) return fail(SAWATTN_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
            if (workspace_bytes < 2 * in_bytes)
                return fail(SAWATTN_ERR_INVALID_ARG, "workspace is smaller than attn_fwd_workspace_bytes reports");
            const uintptr_t w0 = (uintptr_t)workspace, w1 = w0 + 2 * in_bytes;
            for (const void* in : {Q, K, V}) {
                const uintptr_t i0 = (uintptr_t)in, i1 = i0 + in_bytes;
                if (w0 < i1 && i0 < w1) return fail(SAWATTN_ERR_INVALID_ARG, "workspace must not overlap Q, K, V or O");
            }
            if (w0 < o1 && o0 < w1) return fail(SAWATTN_ERR_INVALID_ARG, "workspace must not overlap Q, K, V or O");
        }
    }

    Params p;
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.trace = trace; p.trace_count = trace_count;
    p.N = N;
    p.o_dtype = o_dtype;
    p.sawtooth = scan_order == SAWATTN_SCAN_SAWTOOTH;
    p.negate_q = scale < 0.f;
    p.q_bf16 = converted;
    {
        p.stream_o = sched.qo_streaming == 1 || sched.qo_streaming == 3;
        p.stream_q = sched.qo_streaming == 2 || sched.qo_streaming == 3;
    }
    // Never zero: the kernels mask a key by giving it the score -inf and rely on -inf * c = -inf.  At this floor
    // every finite score times c is below 2^-60 in magnitude, so scale = 0 still gives exp2(0) = 1 for every visible key.
    p.c = std::fmax((float)(std::fabs((double)scale) * 1.4426950408889634074), 1e-30f);
    p.sched = sched;
    p.max_local = sched.local_iters;
    const int grid = sched.grid;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool bf = in_dtype == SAWATTN_BF16, ca = causal != 0;
    if (converted) {
        const size_t chunks = (size_t)B * H * N * d / 8;
        u4* K16 = static_cast<u4*>(workspace);
        u4* V16 = K16 + chunks;
        const unsigned blocks = (unsigned)std::min<size_t>((chunks + 255) / 256, 256 * 16);
        hipLaunchKernelGGL(bf16_to_f16_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const u4*>(K),
                           static_cast<const u4*>(V), K16, V16, chunks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(SAWATTN_ERR_RUNTIME, "conversion kernel launch failed");
        p.K = K16;
        p.V = V16;
    }
    if (sched.tile_q > kTileQ) {
        if (bf && !converted) return ca ? launch<128, true, true, 2>(p, grid, stream) : launch<128, true, false, 2>(p, grid, stream);
        return ca ? launch<128, false, true, 2>(p, grid, stream) : launch<128, false, false, 2>(p, grid, stream);
    }
    if (sched.tile_q < kTileQ) {   // 64-row tiles: the two halves of the K/V scan at once
        if (d == 128) {
            if (bf) return ca ? launch<128, true, true, 1, true>(p, grid, stream) : launch<128, true, false, 1, true>(p, grid, stream);
            return ca ? launch<128, false, true, 1, true>(p, grid, stream) : launch<128, false, false, 1, true>(p, grid, stream);
        }
        if (bf) return ca ? launch<64, true, true, 1, true>(p, grid, stream) : launch<64, true, false, 1, true>(p, grid, stream);
        return ca ? launch<64, false, true, 1, true>(p, grid, stream) : launch<64, false, false, 1, true>(p, grid, stream);
    }
    if (d == 128) {
        if (bf) return ca ? launch<128, true, true, 1>(p, grid, stream) : launch<128, true, false, 1>(p, grid, stream);
        return ca ? launch<128, false, true, 1>(p, grid, stream) : launch<128, false, false, 1>(p, grid, stream);
    }
    if (bf) return ca ? launch<64, true, true, 1>(p, grid, stream) : launch<64, true, false, 1>(p, grid, stream);
    return ca ? launch<64, false, true, 1>(p, grid, stream) : launch<64, false, false, 1>(p, grid, stream);
}

// ---- scratch memory of attn_fwd_static: a fixed array in device memory instead of a caller's workspace.
// Every GPU the library runs on holds its own copy at its own address; host code never uses the array's name as
// an address, only what hipGetSymbolAddress returned for the device that was current.
constexpr size_t kStaticScratchBytes = (size_t)SAWATTN_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return fail(SAWATTN_ERR_RUNTIME, "cannot query the current device (or its index is 64 or more)");
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            char msg[200];
            std::snprintf(msg, sizeof msg, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
            return fail(SAWATTN_ERR_RUNTIME, msg);
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SAWATTN_OK;
}

// Argument checks shared by the queries that launch nothing.
int check_query(int B, int H, int N, int d, int in_dtype) {
    if (in_dtype != SAWATTN_F16 && in_dtype != SAWATTN_BF16)
        return fail(SAWATTN_ERR_INVALID_ARG, "in_dtype must be SAWATTN_F16 or SAWATTN_BF16");
    return check_shape(B, H, N, d);
}

}  // namespace sawattn

extern "C" {

int attn_fwd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale, int causal,
             int scan_order, int in_dtype, int o_dtype, void* hip_stream) {
    return sawattn::run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, nullptr, nullptr,
                        nullptr);
}

int attn_fwd_variant(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                     int causal, int scan_order, int in_dtype, int o_dtype, void* hip_stream,
                     const sawattn_variant* variant, int32_t* trace, int32_t* trace_count) {
    return sawattn::run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, variant, trace,
                        trace_count);
}

int attn_fwd_workspace(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                       int causal, int scan_order, int in_dtype, int o_dtype, void* hip_stream,
                       const sawattn_variant* variant, int32_t* trace, int32_t* trace_count, void* workspace,
                       size_t workspace_bytes) {
    return sawattn::run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, variant, trace,
                        trace_count, workspace, workspace_bytes);
}

int attn_fwd_workspace_bytes(int B, int H, int N, int d, int causal, int in_dtype, const sawattn_variant* variant,
                             size_t* bytes, sawattn_launch_info* info) {
    using namespace sawattn;
    if (!bytes) return fail(SAWATTN_ERR_INVALID_ARG, "bytes must be non-null");
    int rc = check_query(B, H, N, d, in_dtype);
    if (rc != SAWATTN_OK) return rc;
    Schedule s;
    bool use = false;
    rc = workspace_schedule(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &s, &use);
    if (rc != SAWATTN_OK) return rc;
    if (!use) {
        rc = schedule_for(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &s);
        if (rc != SAWATTN_OK) return rc;
    }
    *bytes = use ? (size_t)B * H * N * d * 4 : 0;
    if (info) fill_info(s, d, info);
    return SAWATTN_OK;
}

int attn_fwd_static(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                    int causal, int scan_order, int in_dtype, int o_dtype, void* hip_stream) {
    using namespace sawattn;
    size_t need = 0;
    int rc = attn_fwd_workspace_bytes(B, H, N, d, causal, in_dtype, nullptr, &need, nullptr);
    if (rc != SAWATTN_OK) return rc;
    if (need > kStaticScratchBytes) {
        char msg[200];
        std::snprintf(msg, sizeof msg, "attn_fwd_static: this problem needs %zu bytes of scratch, the fixed array holds %zu "
                      "(4*B*H*N*d must not exceed it)", need, kStaticScratchBytes);
        return fail(SAWATTN_ERR_UNSUPPORTED, msg);
    }
    void* ws = nullptr;
    if (need) {
        rc = static_scratch(&ws);
        if (rc != SAWATTN_OK) return rc;
    }
    return run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, nullptr, nullptr, nullptr,
               ws, need);
}

int attn_fwd_variant_launch_info(int B, int H, int N, int d, int causal, int in_dtype, const sawattn_variant* variant,
                                 sawattn_launch_info* out) {
    using namespace sawattn;
    if (!out) return fail(SAWATTN_ERR_INVALID_ARG, "out must be non-null");
    int rc = check_query(B, H, N, d, in_dtype);
    if (rc != SAWATTN_OK) return rc;
    Schedule s;
    rc = schedule_for(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &s);
    if (rc != SAWATTN_OK) return rc;
    fill_info(s, d, out);
    return SAWATTN_OK;
}

int attn_fwd_launch_info(int B, int H, int N, int d, int causal, int scan_order, int in_dtype, sawattn_launch_info* out) {
    if (scan_order != SAWATTN_SCAN_CYCLIC && scan_order != SAWATTN_SCAN_SAWTOOTH)
        return sawattn::fail(SAWATTN_ERR_INVALID_ARG, "scan_order must be SAWATTN_SCAN_CYCLIC or SAWATTN_SCAN_SAWTOOTH");
    return attn_fwd_variant_launch_info(B, H, N, d, causal, in_dtype, nullptr, out);
}

int attn_fwd_plan(int B, int H, int N, int d, int causal, int scan_order, int in_dtype, const sawattn_variant* variant,
                  int32_t* trace, int32_t* trace_count) {
    using namespace sawattn;
    if (!trace || !trace_count) return fail(SAWATTN_ERR_INVALID_ARG, "trace and trace_count must be non-null");
    if (scan_order != SAWATTN_SCAN_CYCLIC && scan_order != SAWATTN_SCAN_SAWTOOTH)
        return fail(SAWATTN_ERR_INVALID_ARG, "scan_order must be SAWATTN_SCAN_CYCLIC or SAWATTN_SCAN_SAWTOOTH");
    int rc = check_query(B, H, N, d, in_dtype);
    if (rc != SAWATTN_OK) return rc;
    Schedule s;
    rc = schedule_for(B, H, N, d, causal != 0, in_dtype == SAWATTN_BF16, variant, &s);
    if (rc != SAWATTN_OK) return rc;
    // the kernel's outer loop, one workgroup at a time
    for (int wg = 0; wg < s.grid; ++wg) {
        int local = 0;
        for (int it = 0; it < s.local_iters; ++it) {
            const Work w = decode_work(s, wg, it, causal != 0, scan_order == SAWATTN_SCAN_SAWTOOTH);
            if (w.tile < 0) continue;
            const int nkv = visible_kv_tiles(s, w.tile, N, causal != 0);
            int32_t* rec = trace + ((size_t)wg * s.local_iters + local) * 4;
            rec[0] = w.head; rec[1] = w.tile; rec[2] = w.backward ? nkv - 1 : 0; rec[3] = w.backward ? 0 : nkv - 1;
            ++local;
        }
        trace_count[wg] = local;
    }
    return SAWATTN_OK;
}

const char* attn_last_error(void) { return sawattn::g_err; }
int attn_version(void) { return 212; }
const char* sawattn_last_error(void) { return attn_last_error(); }
int sawattn_version(void) { return attn_version(); }

}  // extern "C"
