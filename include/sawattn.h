/*
 * sawattn -- FlashAttention forward with Sawtooth Wavefront Reordering for AMD MI355X (gfx950).
 *
 * C ABI of libsawattn.so.  Plain pointers and sizes only; every pointer named "device" must be a
 * HIP device pointer on the current device, every pointer named "host" an ordinary host pointer.
 * No function here throws, aborts, allocates device memory or synchronises the device, unless its
 * comment says otherwise.  All functions return SAWATTN_OK or an error code; the text of the last
 * error on the calling thread is available from attn_last_error().
 *
 * The four entry points a caller of the method needs are attn_fwd, attn_fwd_launch_info, attn_last_error
 * and attn_version.  The others serve the studies of the paper's Sec. 3 and Sec. 4.3 (launch variants,
 * recorded schedules), bfloat16 inputs with caller-provided or built-in scratch memory, and older names.
 */
#ifndef SAWATTN_H
#define SAWATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SAWATTN_OK = 0,
    SAWATTN_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, non-positive size, bad enum, overflow */
    SAWATTN_ERR_UNSUPPORTED = 2,   /* head dimension other than 64 or 128; a variant the problem does not admit */
    SAWATTN_ERR_RUNTIME = 3        /* the HIP runtime refused the launch */
};

/* Order in which a workgroup walks the K/V tiles of one query tile (paper Sec. 4, Alg. 4). */
enum {
    SAWATTN_SCAN_CYCLIC = 0,       /* always ascending */
    SAWATTN_SCAN_SAWTOOTH = 1      /* ascending on even, descending on odd rounds over one head's K/V */
};

enum {
    SAWATTN_F16 = 0,               /* IEEE binary16 */
    SAWATTN_BF16 = 1,              /* bfloat16 */
    SAWATTN_F32 = 2                /* IEEE binary32; allowed for the output only */
};

/* The same constants under the short prefix. */
enum {
    ATTN_OK = SAWATTN_OK, ATTN_ERR_INVALID_ARG = SAWATTN_ERR_INVALID_ARG,
    ATTN_ERR_UNSUPPORTED = SAWATTN_ERR_UNSUPPORTED, ATTN_ERR_RUNTIME = SAWATTN_ERR_RUNTIME,
    ATTN_SCAN_CYCLIC = SAWATTN_SCAN_CYCLIC, ATTN_SCAN_SAWTOOTH = SAWATTN_SCAN_SAWTOOTH,
    ATTN_F16 = SAWATTN_F16, ATTN_BF16 = SAWATTN_BF16, ATTN_F32 = SAWATTN_F32
};

/*
 * attn_fwd -- O = softmax(Q K^T * scale) V  (paper Sec. 2.2, Eq. 1), computed tile by tile with an
 * online softmax (Alg. 1) by persistent workgroups (Alg. 2) that scan K/V in `scan_order` (Alg. 4); where
 * heads are short and come several to an XCD, by one workgroup per query tile instead (Alg. 3; see
 * SAWATTN_LAUNCH_AUTO below).
 *
 *   Q, K, V  device, read only.  Contiguous [B, H, N, d], d fastest, element type `in_dtype`
 *            (SAWATTN_F16 or SAWATTN_BF16), 16-byte aligned.  Query and key sequences both have
 *            length N; each (batch, head) pair is an independent attention problem.
 *   O        device, written.  Contiguous [B, H, N, d], element type `o_dtype` (F16, BF16 or F32),
 *            16-byte aligned.  Every element is overwritten.  Must not overlap Q, K or V.
 *   B, H, N  >= 1.   d must be 64 or 128.   B*H*N*d must be below 2^40 and B*H*ceil(N/128) below 2^31.
 *   scale    any finite float (1/sqrt(d) in the paper); the scores are multiplied by it.
 *   causal   0: every key is visible;  non-zero: key j is visible to query i iff j <= i.
 *   scan_order  SAWATTN_SCAN_CYCLIC or SAWATTN_SCAN_SAWTOOTH.  Both give the same O up to the
 *            rounding of a different fp32 summation order.
 *   hip_stream  a hipStream_t (NULL = the default stream).  The kernel is enqueued there and the call
 *            returns without waiting; the caller keeps all buffers alive until the stream has drained.
 *
 * Arithmetic: 16-bit inputs are multiplied exactly and accumulated in fp32 on the matrix cores; `scale` is
 * applied to the fp32 scores (no input is rounded again); the
 * running maximum, the running sum and the output accumulator are fp32; the probabilities are
 * rounded to binary16 before the second contraction (for bf16 inputs V is converted to binary16 on
 * the way into LDS, which is exact for |v| in [2^-14, 65504] -- larger bf16 values of V are not
 * supported).  The caller owns every buffer.  Besides the per-thread error text the library holds
 * one piece of device state: eight sets of eight 32-bit arrival counters (one per XCD) with which the
 * workgroups of an XCD wait for each other, for a bounded time, before they move on to the next
 * head, so that they keep streaming the same K/V through their shared L2.  A launch that has more
 * than one head per XCD takes the next set in turn and clears it first (a one-block kernel on the
 * same stream), so launches that overlap on one device -- other streams, other host threads -- leave
 * each other alone unless eight or more are in flight.  The counters steer timing only, never
 * results, and no wait is unbounded: at worst (the other workgroups of an XCD not running at all, or
 * nine overlapping launches) a workgroup waits about 8 ms at a head boundary and carries on.
 *
 * Errors: INVALID_ARG / UNSUPPORTED as listed above (nothing is launched); RUNTIME if the launch
 * fails.  Safe to call from several host threads.
 */
int attn_fwd(const void* Q, const void* K, const void* V, void* O,
             int B, int H, int N, int d, float scale, int causal, int scan_order,
             int in_dtype, int o_dtype, void* hip_stream);

/*
 * Launch variants (paper Sec. 2.2 Alg. 2 and Alg. 3, Sec. 3.4, Sec. 4.3), selectable so that they can be
 * measured against the default.  All compute the same O; only which workgroup takes which query tile,
 * when, and in which direction it walks K/V differs.
 */
enum {
    SAWATTN_LAUNCH_PERSISTENT = 0, /* Alg. 2: a fixed set of workgroups loops over the query tiles */
    SAWATTN_LAUNCH_GRID = 1,       /* Alg. 3: one workgroup per `tiles_per_workgroup` consecutive query
                                      tiles, handed to the hardware dispatcher */
    SAWATTN_LAUNCH_AUTO = 2        /* what attn_fwd does: PERSISTENT, except where a head has fewer query tiles than
                                      an XCD holds workgroups and an XCD has two or more heads to go through --
                                      then GRID with one tile per workgroup, so that the tiles of several heads run
                                      side by side (under the causal mask only for heads of at most half that many
                                      tiles, and with two heads per XCD only if all their tiles fit the XCD's 32
                                      compute units at once; with slots_per_domain or the linear decode given:
                                      PERSISTENT) */
};
enum {
    SAWATTN_DECODE_DOMAIN = 0,     /* work is dealt out per XCD (one L2 each): the workgroups of an XCD
                                      share one head's K/V at a time; causal heads start with their
                                      longest tiles */
    SAWATTN_DECODE_LINEAR = 1      /* as printed: one linear index over (batch, head, tile), tile fastest;
                                      persistent workgroup k takes k, k+G, k+2G, ... */
};
typedef struct sawattn_variant {
    int launch;              /* SAWATTN_LAUNCH_* (0 = PERSISTENT; attn_fwd itself runs AUTO) */
    int decode;              /* SAWATTN_DECODE_* */
    int slots_per_domain;    /* persistent launch: at most this many workgroups per XCD, so G = 8 * slots
                                (Sec. 3.4's resident-CTA sweep): 1..64, or 1..96 for d = 64, where three
                                workgroups fit a CU; 0 = default (that maximum).  Ignored by the grid launch. */
    int tiles_per_workgroup; /* grid launch: 1, or 2 = forward over the first tile and, with the sawtooth
                                order, backward over the second (Sec. 4.3's step-2 alternation);
                                0 = default (2; 1 where AUTO picks the grid launch).  Ignored by the persistent launch. */
    int rows_per_wavefront;  /* 32: a workgroup takes 128 query rows (two or three workgroups per CU);
                                64 (d = 128 only; UNSUPPORTED otherwise): 256 rows, one workgroup per CU (at
                                most 32 per XCD), every K/V fragment read from LDS feeds two MFMAs; same
                                arithmetic as the 32-row kernel;
                                0 = default: 64 for d = 128, slots_per_domain <= 32 and sequences long enough
                                that every workgroup of an XCD gets at least one 256-row tile of a head (nearly
                                two under the causal mask) and the rounds of 32 tiles are well filled: with
                                q = ceil(ceil(N/256) / parts_per_head), q >= 32 (56) and q at least 4/5 (3/4) of
                                32 * ceil(q/32); else 32. */
    int align_rounds;        /* persistent launch with the per-XCD decode: 0 = the workgroups of an XCD wait for each
                                other between heads only (and only where they finish a head together); 1 = after
                                every round as well, which holds them in the lockstep Sec. 3.4 assumes at a cost in
                                time.  For measuring what the scan order can save at best.  Ignored otherwise. */
    int kv_halves;           /* 1: a workgroup's wavefronts each own query rows and walk the whole scan;
                                2 (32 rows per wavefront; UNSUPPORTED with 64): a workgroup
                                takes 64 query rows, two wavefronts walk the first half of the full, unmasked
                                K/V tiles of the scan and two the second half, at once, and the two partial
                                softmax results are merged (Alg. 1's update applied to two partial results
                                instead of one tile at a time); an odd tile and the masked ones are taken by the
                                first two wavefronts alone -- for problems too small to occupy the chip, where
                                the length of one wavefront's walk is the launch time;
                                0 = default: 2 where it is supported and B*H*ceil(N/128) is at most 128 (d = 128),
                                or, with d = 64 and N >= 2048, 384 (512 under the causal mask); else 1. */
    int qo_streaming;        /* how the rows touched once per query tile pass the L2.  3: Q tiles are brought in and O tiles
                                written out through LDS, whole 128-byte lines per instruction, marked non-temporal, so
                                that at a round boundary they do not displace the K/V tail the sawtooth order
                                (Sec. 3.4) is about to find in the L2; 1: O only; 2: Q only; 4: neither -- every lane
                                loads and stores the 8- and 16-byte pieces of the rows it computes with, cached;
                                0 = default: 3 where K and V of a head take at least 2 MiB (half the L2 of an XCD),
                                else 1.  Same values written in every mode. */
} sawattn_variant;
/*
 * Scan direction per variant with SAWATTN_SCAN_SAWTOOTH: persistent + domain decode: parity of the round
 * over the current head (the default); persistent + linear decode: parity of the workgroup's own
 * iteration count (Alg. 4 as printed); grid launch: parity of the tile's position in its workgroup.
 * A NULL variant pointer selects { PERSISTENT, DOMAIN, 0, 0, 0, 0 }, which is what attn_fwd runs.
 */

/*
 * attn_fwd_variant -- attn_fwd under a launch variant, optionally recording the schedule: every
 * workgroup notes which query tile it took at each of its local iterations and in which direction it
 * walked the K/V tiles (paper Sec. 2.2 Alg. 2/3 work decode, Sec. 4 Alg. 4 scan direction).
 *
 *   variant      host, read during the call only; NULL = default.
 *   trace        device, written, or NULL: int32 [grid][max_local_tiles][4] = (b*H + h, query tile
 *                index, first K/V tile visited, last K/V tile visited); grid and max_local_tiles from
 *                attn_fwd_variant_launch_info for the same variant.  Unused records are left untouched.
 *   trace_count  device, written, or NULL (both or neither): int32 [grid], records each workgroup wrote.
 * All other arguments, errors and stream behaviour as attn_fwd; INVALID_ARG for a bad variant field.
 */
int attn_fwd_variant(const void* Q, const void* K, const void* V, void* O,
                     int B, int H, int N, int d, float scale, int causal, int scan_order,
                     int in_dtype, int o_dtype, void* hip_stream,
                     const sawattn_variant* variant, int32_t* trace, int32_t* trace_count);

/* Launch geometry chosen for a problem; filled by attn_fwd_launch_info (host memory). */
typedef struct sawattn_launch_info {
    int tile_q;            /* query rows per workgroup tile */
    int tile_kv;           /* key/value rows per streamed tile */
    int block_threads;     /* threads per workgroup (64-wide wavefronts) */
    int grid;              /* workgroups launched, a multiple of `domains` */
    int lds_bytes;         /* dynamic LDS per workgroup */
    int domains;           /* cache domains (XCDs, one L2 each) the schedule is built for */
    int slots;             /* workgroups per domain = grid / domains */
    int parts_per_head;    /* domains that share one head's query tiles (1 when B*H % 8 == 0) */
    int q_tiles_per_head;  /* ceil(N / tile_q) */
    int max_local_tiles;   /* most query tiles any one workgroup processes */
    int launch;            /* SAWATTN_LAUNCH_PERSISTENT or SAWATTN_LAUNCH_GRID: which of the two runs */
    int tiles_per_workgroup; /* grid launch: consecutive query tiles per workgroup (1 with the persistent launch) */
    int qo_streaming;        /* 1, 2, 3 or 4 as in sawattn_variant: how Q and O tiles pass the L2 in this launch */
} sawattn_launch_info;

/*
 * attn_fwd_workspace -- attn_fwd_variant with scratch memory from the caller (paper Sec. 2.2, Alg. 1: the same
 * kernel; the scratch only changes the element type K and V are streamed in).  On bfloat16 inputs the kernels
 * convert V to binary16 on its way into LDS, in every workgroup that streams it; the 64-rows-per-wavefront kernel,
 * whose one wavefront per SIMD has no instruction slots to spare, pays for that (about 5 % on long sequences).
 * Given a workspace, and where that kernel is chosen (d = 128, sequence long enough; or
 * variant.rows_per_wavefront = 64), the call first writes binary16 copies of K and V into the workspace with one
 * extra kernel on the same stream and then runs the 64-row kernel on them, converting Q as it is loaded.  The
 * copies are exact for bfloat16 magnitudes in [2^-14, 65504] and rounded to binary16 subnormals below (absolute
 * error under 2^-25); larger Q, K or V values are not supported on this path (V has that limit in attn_fwd as
 * well).  In every other case the call is attn_fwd_variant and the workspace is not touched.
 *
 *   workspace        device, written, 16-byte aligned, must not overlap Q, K, V or O; may be NULL (then this is
 *                    attn_fwd_variant).  Only used during the kernels this call enqueues.
 *   workspace_bytes  its size; at least what attn_fwd_workspace_bytes reports, else INVALID_ARG.
 * Nothing is allocated by the library.  All other arguments, errors and stream behaviour as attn_fwd_variant;
 * the launch geometry (for trace) is what attn_fwd_workspace_bytes reports in `info`.
 */
int attn_fwd_workspace(const void* Q, const void* K, const void* V, void* O,
                       int B, int H, int N, int d, float scale, int causal, int scan_order,
                       int in_dtype, int o_dtype, void* hip_stream,
                       const sawattn_variant* variant, int32_t* trace, int32_t* trace_count,
                       void* workspace, size_t workspace_bytes);

/*
 * attn_fwd_workspace_bytes -- how much workspace attn_fwd_workspace would use for a problem: 4*B*H*N*d bytes
 * (binary16 copies of K and V) where the conversion path applies, 0 where it does not (then a workspace changes
 * nothing).  No passage of the paper corresponds to it: it is the sizing helper of attn_fwd_workspace.  `bytes`
 * and `info` are host memory; `info` may be NULL, else it receives the launch geometry of the kernel
 * attn_fwd_workspace would run.  Validation as attn_fwd_variant_launch_info.  Launches nothing.
 */
int attn_fwd_workspace_bytes(int B, int H, int N, int d, int causal, int in_dtype,
                             const sawattn_variant* variant, size_t* bytes, sawattn_launch_info* info);

/*
 * attn_fwd_static -- attn_fwd for callers that may not allocate device memory and have no workspace to lend:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is attn_fwd_workspace
 * with the default variant and no trace, the workspace being a fixed array of SAWATTN_STATIC_SCRATCH_BYTES in
 * the library's device data (each GPU the library runs on holds its own copy from the time the library's code is
 * loaded there until the process ends).  The call itself allocates and frees nothing, on the host or the device.
 *
 *   Arguments, stream behaviour and errors as attn_fwd.  In addition UNSUPPORTED, with the sizes in the error
 *   text, if the problem would use more scratch than the array holds, i.e. if attn_fwd_workspace_bytes reports
 *   more than SAWATTN_STATIC_SCRATCH_BYTES (bfloat16 inputs on the conversion path: 4*B*H*N*d bytes); problems
 *   that use no scratch (binary16 inputs, short sequences, d = 64) have no size limit beyond attn_fwd's.
 *   The first call on a device looks up the array's address there (hipGetSymbolAddress) and sets a kernel
 *   attribute; make one call outside any stream capture first.
 *   Every call on one GPU uses the same array, whose contents are overwritten by each call that needs it (nothing
 *   in it has to start out zero): calls that overlap in time on one GPU -- two streams, two host threads -- race on
 *   it and give wrong results; calls on one stream, or ordered by events, are safe.
 */
#define SAWATTN_STATIC_SCRATCH_BYTES (64u << 20)
int attn_fwd_static(const void* Q, const void* K, const void* V, void* O,
                    int B, int H, int N, int d, float scale, int causal, int scan_order,
                    int in_dtype, int o_dtype, void* hip_stream);

/*
 * attn_fwd_launch_info -- report the geometry attn_fwd would use (paper Sec. 2.2, Alg. 2: grid size and work
 * decode; Sec. 3.4: workgroups per cache domain).  `out` is host memory.  Validates B, H, N, d, scan_order and
 * in_dtype like attn_fwd (the geometry does not depend on the scan order).  Launches nothing.
 */
typedef sawattn_launch_info attn_launch_info;
int attn_fwd_launch_info(int B, int H, int N, int d, int causal, int scan_order, int in_dtype,
                         attn_launch_info* out);

/*
 * attn_fwd_variant_launch_info -- the same for attn_fwd_variant (paper Sec. 2.2, Alg. 2 / Alg. 3); `variant` is
 * host memory, NULL = the default, and is validated like attn_fwd_variant does.  Launches nothing.
 */
int attn_fwd_variant_launch_info(int B, int H, int N, int d, int causal, int in_dtype,
                                 const sawattn_variant* variant, sawattn_launch_info* out);

/*
 * attn_fwd_plan -- the schedule attn_fwd_variant would run, computed on the host from the same work
 * decode the kernel uses (paper Sec. 2.2 Alg. 2/3, Sec. 4 Alg. 4).  Launches nothing and needs no GPU.
 *
 *   variant      host or NULL, as for attn_fwd_variant.
 *   trace        host, written: int32 [grid][max_local_tiles][4], same record layout as
 *                attn_fwd_variant; unused records are left untouched.
 *   trace_count  host, written: int32 [grid].
 * B, H, N, d, causal, scan_order, in_dtype and the variant are validated like attn_fwd_variant.
 */
int attn_fwd_plan(int B, int H, int N, int d, int causal, int scan_order, int in_dtype,
                  const sawattn_variant* variant, int32_t* trace, int32_t* trace_count);

/* Text of the last error raised on the calling thread ("" if none).  Static storage, never NULL. */
const char* attn_last_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int attn_version(void);

/* Older names of the two functions above. */
const char* sawattn_last_error(void);
int sawattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SAWATTN_H */
