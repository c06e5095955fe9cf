// FlashAttention forward for gfx950 with a selectable K/V scan order (cyclic or sawtooth).
//
// One workgroup = 4 wavefronts = one 128-row query tile (paper Sec. 2.2, Alg. 1); wavefront w owns
// query rows 32w..32w+31 of the tile and keeps them in registers for the whole inner loop.  K and V
// are streamed in 64-row tiles through two LDS buffers each (global -> registers -> LDS, the next
// tile in flight while the current one is used).
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
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "sawattn.h"
#include "schedule.h"

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
    int max_local;
    float c;               // |scale| * log2(e): scores are handled in the log2 domain
    Schedule sched;
};

template <int D>
struct Geo {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kStride = kRowBytes + 16;           // LDS row pitch, padded against bank conflicts
    static constexpr int kTileBytes = kTileKV * kStride;     // one K or V tile in LDS
    static constexpr int kChunksPerRow = D / 8;              // 16-byte chunks per row
    static constexpr int kChunksPerThread = kTileKV * kChunksPerRow / kThreads;
    static constexpr int kLdsBytes = 4 * kTileBytes;         // K0 K1 V0 V1
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

template <int D>
__device__ __forceinline__ void load_tile(const char* base, int kv0, int N, int tid, u4 (&reg)[Geo<D>::kChunksPerThread]) {
#pragma unroll
    for (int i = 0; i < Geo<D>::kChunksPerThread; ++i) {
        int id = tid + i * kThreads;
        int row = id / Geo<D>::kChunksPerRow, cc = id % Geo<D>::kChunksPerRow;
        u4 v = {0u, 0u, 0u, 0u};
        if (kv0 + row < N) v = *reinterpret_cast<const u4*>(base + (size_t)(kv0 + row) * Geo<D>::kRowBytes + cc * 16);
        reg[i] = v;
    }
}

template <int D, bool CONVERT>
__device__ __forceinline__ void store_tile(char* lds, int tid, const u4 (&reg)[Geo<D>::kChunksPerThread]) {
#pragma unroll
    for (int i = 0; i < Geo<D>::kChunksPerThread; ++i) {
        int id = tid + i * kThreads;
        int row = id / Geo<D>::kChunksPerRow, cc = id % Geo<D>::kChunksPerRow;
        u4 v = reg[i];
        if constexpr (CONVERT) v = bf16x8_to_f16x8(v);
        *reinterpret_cast<u4*>(lds + row * Geo<D>::kStride + cc * 16) = v;
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One query tile (Alg. 1 body): rows [t*128, t*128+128) of head `hh`, K/V tiles j0, j0+step, ... (nkv of them).
template <int D, bool BF16, bool CAUSAL>
__device__ __forceinline__ void process_q_tile(const Params& p, int hh, int t, int j0, int step, int nkv, char* smem) {
    using G = Geo<D>;
    constexpr int KS = D / 16;    // MFMA steps along d for S^T
    constexpr int DB = D / 32;    // 32-row blocks of O^T
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, ln = lane & 31;
    const int N = p.N;
    const size_t head_off = (size_t)hh * N * G::kRowBytes;
    const char* Qh = static_cast<const char*>(p.Q) + head_off;
    const char* Kh = static_cast<const char*>(p.K) + head_off;
    const char* Vh = static_cast<const char*>(p.V) + head_off;
    char* Kl[2] = {smem, smem + G::kTileBytes};
    char* Vl[2] = {smem + 2 * G::kTileBytes, smem + 3 * G::kTileBytes};

    const int qw0 = t * kTileQ + wave * 32;   // first query row of this wavefront
    const int qrow = qw0 + ln;                // this lane's query row (column of S^T)
    const bool wave_has_rows = qw0 < N;

    // Q^T as B operand: lane holds Q[qrow][16*ks + 8*g .. +7]
    u4 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        u4 v = {0u, 0u, 0u, 0u};
        if (qrow < N) v = *reinterpret_cast<const u4*>(Qh + (size_t)qrow * G::kRowBytes + ks * 32 + g * 16);
        if (p.negate_q) { v[0] ^= 0x80008000u; v[1] ^= 0x80008000u; v[2] ^= 0x80008000u; v[3] ^= 0x80008000u; }
        qf[ks] = v;
    }

    f16v o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float M = -INFINITY;   // running max of score*c (log2 domain)
    float L = 0.f;         // this lane's partial running sum
    const float c = p.c;

    u4 kreg[G::kChunksPerThread], vreg[G::kChunksPerThread];
    load_tile<D>(Kh, j0 * kTileKV, N, tid, kreg);
    load_tile<D>(Vh, j0 * kTileKV, N, tid, vreg);
    store_tile<D, false>(Kl[0], tid, kreg);
    store_tile<D, BF16>(Vl[0], tid, vreg);
    __syncthreads();

    // per-lane byte offsets inside a tile
    const int k_off = ln * G::kStride + g * 16;
    const int v_off = (4 * g + ((lane & 15) >> 2)) * G::kStride + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    for (int it = 0; it < nkv; ++it) {
        const int cur = it & 1;
        const int j = j0 + it * step;
        const int kv0 = j * kTileKV;
        const bool more = it + 1 < nkv;
        if (more) {
            load_tile<D>(Kh, (j + step) * kTileKV, N, tid, kreg);
            load_tile<D>(Vh, (j + step) * kTileKV, N, tid, vreg);
        }
        const bool active = wave_has_rows && (!CAUSAL || kv0 <= qw0 + 31);
        if (active) {
            // ---- S^T = K_j Q_i^T : two 32(kv) x 32(q) blocks
            f16v s[2];
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[0][r] = 0.f; s[1][r] = 0.f; }
            const char* kl = Kl[cur] + k_off;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                u4 a0 = *reinterpret_cast<const u4*>(kl + ks * 32);
                u4 a1 = *reinterpret_cast<const u4*>(kl + 32 * G::kStride + ks * 32);
                s[0] = mfma_16bit<BF16>(a0, qf[ks], s[0]);
                s[1] = mfma_16bit<BF16>(a1, qf[ks], s[1]);
            }
            // ---- mask: keys beyond N, and keys after the query under the causal mask
            const bool need_mask = (kv0 + kTileKV > N) || (CAUSAL && kv0 + kTileKV - 1 > qw0);
            unsigned masked = 0u;
            if (need_mask) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int kv = kv0 + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3);
                        bool m = (kv >= N) || (CAUSAL && kv > qrow);
                        if (m) { masked |= 1u << (16 * b + r); s[b][r] = -INFINITY; }
                    }
            }
            // ---- online softmax (log2 domain)
            float mx = s[0][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float Mnew = fmaxf(M, mx * c);
            const float Muse = (Mnew == -INFINITY) ? 0.f : Mnew;
            const float alpha = fast_exp2(M - Muse);
            M = Mnew;
            float lsum = 0.f;
            u4 pf[4];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                float pv[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float x = fast_exp2(__builtin_fmaf(s[b][r], c, -Muse));
                    if (need_mask && ((masked >> (16 * b + r)) & 1u)) x = 0.f;
                    pv[r] = x;
                    lsum += x;
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    u4 w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        f2 x2 = {pv[8 * h + 2 * i], pv[8 * h + 2 * i + 1]};
                        w[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(x2, h2));
                    }
                    pf[2 * b + h] = w;
                }
            }
            L = L * alpha + lsum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            // ---- O^T += V_j^T P^T
            const char* vl = Vl[cur] + v_off;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const char* a = vl + (16 * ks) * G::kStride + db * 64;
                    s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(a));
                    s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s4))(a + 8 * G::kStride));
                    s8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, av), __builtin_bit_cast(h8, pf[ks]), o[db], 0, 0, 0);
                }
            }
        }
        if (more) {
            store_tile<D, false>(Kl[cur ^ 1], tid, kreg);
            store_tile<D, BF16>(Vl[cur ^ 1], tid, vreg);
        }
        __syncthreads();
    }

    // ---- epilogue: O_i = acc / l  (the division Alg. 1 leaves implicit; Eq. 1 fixes it)
    const float Ltot = L + __shfl_xor(L, 32, 64);
    const float inv = 1.0f / Ltot;
    if (qrow < N) {
        const size_t orow = ((size_t)hh * N + qrow) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f4 v = {o[db][4 * rq] * inv, o[db][4 * rq + 1] * inv, o[db][4 * rq + 2] * inv, o[db][4 * rq + 3] * inv};
                const size_t col = 32 * db + 8 * rq + 4 * g;
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

template <int D, bool BF16, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(Params p) {
    extern __shared__ __align__(16) char smem[];
    const Schedule& s = p.sched;
    const int domain = blockIdx.x % kDomains;
    const int slot = blockIdx.x / kDomains;
    int round_counter = 0;   // rounds this domain has started (same value in all its workgroups)
    int local = 0;           // query tiles this workgroup has processed (Alg. 4's i_local)
    for (int cs = 0; cs < s.chunks_per_domain; ++cs) {
        for (int r = 0; r < s.rounds_per_chunk; ++r, ++round_counter) {
            int hh;
            const int t = decode_tile(s, domain, slot, cs, r, CAUSAL, &hh);
            if (t < 0) continue;
            const int nkv = visible_kv_tiles(s, t, p.N, CAUSAL);
            const bool backward = p.sawtooth && (round_counter & 1);
            const int j0 = backward ? nkv - 1 : 0;
            const int step = backward ? -1 : 1;
            if (p.trace && threadIdx.x == 0) {
                int32_t* rec = p.trace + ((size_t)blockIdx.x * p.max_local + local) * 4;
                rec[0] = hh; rec[1] = t; rec[2] = j0; rec[3] = j0 + (nkv - 1) * step;
            }
            process_q_tile<D, BF16, CAUSAL>(p, hh, t, j0, step, nkv, smem);
            ++local;
        }
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
    out->tile_q = kTileQ;
    out->tile_kv = kTileKV;
    out->block_threads = kThreads;
    out->grid = kDomains * s.slots;
    out->lds_bytes = d == 128 ? Geo<128>::kLdsBytes : Geo<64>::kLdsBytes;
    out->domains = kDomains;
    out->slots = s.slots;
    out->parts_per_head = s.parts;
    out->q_tiles_per_head = s.q_tiles;
    out->max_local_tiles = s.chunks_per_domain * s.rounds_per_chunk;
}

template <int D, bool BF16, bool CAUSAL>
int launch(const Params& p, int grid, hipStream_t stream) {
    auto kern = attn_fwd_kernel<D, BF16, CAUSAL>;
    static thread_local bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                Geo<D>::kLdsBytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(SAWATTN_ERR_RUNTIME, "hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed");
        }
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), Geo<D>::kLdsBytes, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        char msg[200];
        std::snprintf(msg, sizeof msg, "kernel launch failed: %s", hipGetErrorString(e));
        return fail(SAWATTN_ERR_RUNTIME, msg);
    }
    return SAWATTN_OK;
}

int run(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale, int causal,
        int scan_order, int in_dtype, int o_dtype, void* hip_stream, int32_t* trace, int32_t* trace_count) {
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

    Params p;
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.trace = trace; p.trace_count = trace_count;
    p.N = N;
    p.o_dtype = o_dtype;
    p.sawtooth = scan_order == SAWATTN_SCAN_SAWTOOTH;
    p.negate_q = scale < 0.f;
    p.c = (float)(std::fabs((double)scale) * 1.4426950408889634074);
    p.sched = make_schedule(B * H, N);
    p.max_local = p.sched.chunks_per_domain * p.sched.rounds_per_chunk;
    const int grid = kDomains * p.sched.slots;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool bf = in_dtype == SAWATTN_BF16, ca = causal != 0;
    if (d == 128) {
        if (bf) return ca ? launch<128, true, true>(p, grid, stream) : launch<128, true, false>(p, grid, stream);
        return ca ? launch<128, false, true>(p, grid, stream) : launch<128, false, false>(p, grid, stream);
    }
    if (bf) return ca ? launch<64, true, true>(p, grid, stream) : launch<64, true, false>(p, grid, stream);
    return ca ? launch<64, false, true>(p, grid, stream) : launch<64, false, false>(p, grid, stream);
}

}  // namespace sawattn

extern "C" {

int attn_fwd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale, int causal,
             int scan_order, int in_dtype, int o_dtype, void* hip_stream) {
    return sawattn::run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, nullptr, nullptr);
}

int attn_fwd_trace(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int d, float scale,
                   int causal, int scan_order, int in_dtype, int o_dtype, void* hip_stream, int32_t* trace,
                   int32_t* trace_count) {
    if (!trace || !trace_count) return sawattn::fail(SAWATTN_ERR_INVALID_ARG, "trace and trace_count must be non-null");
    return sawattn::run(Q, K, V, O, B, H, N, d, scale, causal, scan_order, in_dtype, o_dtype, hip_stream, trace, trace_count);
}

int attn_fwd_launch_info(int B, int H, int N, int d, int causal, sawattn_launch_info* out) {
    (void)causal;
    if (!out) return sawattn::fail(SAWATTN_ERR_INVALID_ARG, "out must be non-null");
    int rc = sawattn::check_shape(B, H, N, d);
    if (rc != SAWATTN_OK) return rc;
    sawattn::fill_info(sawattn::make_schedule(B * H, N), d, out);
    return SAWATTN_OK;
}

const char* sawattn_last_error(void) { return sawattn::g_err; }

int sawattn_version(void) { return 100; }

}  // extern "C"
