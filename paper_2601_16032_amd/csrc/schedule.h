// Work decode shared by the host launcher and the kernel: which workgroup takes which query tile,
// in which round, and in which direction it then walks the K/V tiles.
//
// The paper launches G persistent workgroups that stride over a linear (batch, head, tile) index
// (Sec. 2.2, Alg. 2) and flips the K/V scan direction on every other local iteration (Sec. 4,
// Alg. 4).  The reuse it relies on happens among workgroups that share one L2 (Sec. 3.4).  On
// MI355X that sharing domain is one XCD: the hardware places workgroup `wg` on XCD `wg % 8`, so the
// linear index is decoded per domain:
//
//   * a head's query tiles are split into `parts` interleaved subsets (parts = 8 / gcd(B*H, 8), so
//     1 when B*H is a multiple of 8); chunk c = head*parts + part runs on domain c % 8, and the
//     chunks of one domain run one after another;
//   * inside a chunk the `slots` workgroups of the domain take its tiles in rounds of `slots`
//     consecutive tiles, so all of them stream the same head's K/V at the same time;
//   * a workgroup's odd local iterations (rounds counted across the chunks of its domain) hand
//     the tiles out in reverse slot order, which evens out the causal cost (tile i costs i+1 K/V
//     tiles) inside a head with an even number of rounds and over two heads otherwise; causal
//     chunks start from their longest tile;
//   * the scan direction of a round is the parity of the round index inside its chunk: this is
//     Alg. 4's local-iteration parity restarted at every chunk.  Consecutive rounds of one chunk
//     walk the same K/V, which is where reversing the direction shortens the reuse distance; the
//     first round of a new chunk meets cold K/V whichever way it walks, and walks forward so that
//     causal tiles all start from key 0 together.  Taking the round index rather than a per-
//     workgroup count keeps the whole domain walking one way when a workgroup sits a round out.
#pragma once

#if defined(__HIPCC__)
#define SAW_HD __host__ __device__ inline
#else
#define SAW_HD inline
#endif

namespace sawattn {

constexpr int kTileQ = 128;      // query rows per workgroup tile (twice that in the wide variant)
constexpr int kTileKV = 64;      // key/value rows per streamed tile
constexpr int kThreads = 256;    // 4 wavefronts of 32 query rows each (64 in the wide variant)
constexpr int kDomains = 8;      // XCDs
constexpr int kMaxSlots = 96;    // largest number of workgroups per domain for any tile shape

SAW_HD int gcd_i(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }
SAW_HD int ceil_div_i(long long a, long long b) { return (int)((a + b - 1) / b); }

// Rows per wavefront when the caller leaves the choice open: the wide variant (64 rows, 256-row
// workgroup tiles) for head dimension 128 (either input type) once the steady state dominates, i.e.
// every resident workgroup of a domain gets at least one full-length tile of a head (nearly two under the
// causal mask, where a tile walks half the keys on average), and only if the rounds of 32 tiles are well
// filled: a last round with a few tiles costs this kernel a full round, while the 32-row kernel's workgroups
// run faster when they have their compute unit to themselves.  Measured, 256-row tiles per head and XCD against
// the gain over the 32-row kernel: plain 32: +9 %, 36: -10 %, 40: -9 %, 48: 0, 56: +11 %, 64: +9 %, 72: -5 %,
// 80: +1 %, 88: +12 %, 96: +10 %; causal 48: -4 %, 56: +4 %, 64: +7 %, 72: +2 %, 88: +4 %, 96: +5 %.
SAW_HD int default_rows_per_wavefront(int heads, int N, int d, bool causal, bool bf16) {
    (void)bf16;
    if (d != 128) return 32;
    const int parts = kDomains / gcd_i(heads, kDomains);
    const int wide_tiles = (N + 2 * kTileQ - 1) / (2 * kTileQ);
    const int q = (wide_tiles + parts - 1) / parts;          // tiles of a head on one XCD
    if (q < (causal ? 56 : 32)) return 32;
    const int rounds = (q + 31) / 32;
    // filled to at least 4/5 over all rounds (3/4 under the mask)
    return (causal ? 4 * q >= 3 * 32 * rounds : 5 * q >= 4 * 32 * rounds) ? 64 : 32;
}

// Workgroups per domain that are resident together: 32 CUs per XCD x workgroups per CU.  A head
// dimension of 64 leaves room for three (168 VGPRs per wavefront, 32 KiB LDS per workgroup), 128 for
// two; the wide variant (256-row tiles, up to 512 registers per wavefront, 128 KiB LDS) runs one.
// With 64-row tiles (the two halves of a scan at once, twice the LDS) two fit at d = 64 and one at d = 128.
SAW_HD int resident_slots(int d, int tile_q = kTileQ) {
    if (tile_q > kTileQ) return 32;
    if (tile_q < kTileQ) return d == 64 ? 64 : 32;
    return d == 64 ? 96 : 64;
}

// Small problems: when the 128-row query tiles of the whole problem occupy at most half of the 256 compute units,
// the launch takes as long as one wavefront needs to walk all K/V tiles of a head.  Then a workgroup takes 64 rows
// instead and walks the two halves of the scan at once, two wavefronts each.  At d = 64, where two such workgroups
// fit a compute unit (512 on the chip), it goes on paying for somewhat larger problems, most under the causal mask,
// where the longest tile of a head sets the pace and is the one cut in two.  Measured limits, in 128-row tiles of the
// whole problem: d = 128: 128 (beyond, the 64-row workgroups, one per compute unit, no longer run all at once: up to
// 1.5x slower at 256); d = 64: 384 plain, 512 causal (gains of 3-10 % there, none at 768), and beyond 128 only for
// N >= 2048: a scan of 16 tiles or fewer is too short for its halves to pay for the merge (N = 512: 25 % slower).
// 1 = one scan per workgroup, 2 = two halves.
SAW_HD int default_kv_halves(int heads, int N, int d, bool causal, bool bf16) {
    (void)bf16;
    const long long tiles = (long long)heads * ((N + kTileQ - 1) / kTileQ);
    const int limit = d == 64 && N >= 2048 ? (causal ? 512 : 384) : 128;
    return tiles <= limit ? 2 : 1;
}

// Besides that default, the launch variants the paper describes are kept selectable so that they
// can be measured against it: the literal global stride of Alg. 2 (workgroup k takes the linear
// indices k, k+G, ... with the tile index fastest, direction = parity of its own iteration count,
// Alg. 4 as printed), fewer resident workgroups per domain (Sec. 3.4), and the direct launch of
// Alg. 3 with one workgroup per one or two consecutive query tiles, where the second tile is
// walked backward (the step-2 alternation of Sec. 4.3).
enum { kLaunchPersistent = 0, kLaunchGrid = 1 };

// How the tiles touched once per query tile pass the L2 when the caller leaves it open: O always as whole non-temporal
// lines; Q as well where K and V of a head take at least half the 4 MiB L2 of an XCD -- below that no scan order has
// anything to lose to the Q tiles, and direct loads hide their latency behind the first K/V fetch.
SAW_HD int default_qo_streaming(int N, int d) {
    return (unsigned long long)N * (unsigned)d * 4u >= (2u << 20) ? 3 : 1;
}

// Launch when the caller leaves the choice open.  The persistent hand-out gives one head at a time to the
// workgroups of an XCD, which is what keeps a long head's K/V in one L2; a head with fewer query tiles than the
// XCD holds workgroups then leaves compute units idle, and with several such heads per XCD one after the other
// the launch takes several times longer than it has to (B*H = 128, N = 512, d = 64: 140 us against 17 us).  There
// the direct launch of Alg. 3 with one tile per workgroup is taken: the hardware dispatcher runs the tiles of all
// heads of an XCD side by side, still head by head in workgroup order.  Under the causal mask the persistent
// hand-out has something the dispatcher has not -- it pairs a long tile with a short one per workgroup -- and keeps
// the launch unless the heads are short enough to run two abreast (measured: from half the resident count down),
// or, with only two heads per XCD, unless all their tiles find a compute unit of their own.
SAW_HD int default_launch(int heads, int N, int d, bool causal, int tile_q) {
    const int parts = kDomains / gcd_i(heads, kDomains);
    const int q_tiles = (N + tile_q - 1) / tile_q;
    const int per_part = (q_tiles + parts - 1) / parts;
    const long long chunks = ((long long)heads * parts) / kDomains;
    const int resident = tile_q > kTileQ ? 32 : (tile_q < kTileQ ? (d == 64 ? 64 : 32) : (d == 64 ? 96 : 64));
    if (per_part >= resident || chunks < 2) return kLaunchPersistent;
    if (!causal) return kLaunchGrid;
    if (chunks >= 3) return 2 * per_part <= resident ? kLaunchGrid : kLaunchPersistent;
    return 2 * per_part <= 32 ? kLaunchGrid : kLaunchPersistent;
}
enum { kDecodeDomain = 0, kDecodeLinear = 1 };

struct Schedule {
    int heads;              // B*H
    int tile_q;             // query rows per workgroup tile: kTileQ, or 2*kTileQ in the wide variant
    int q_tiles;            // ceil(N / tile_q)
    int kv_tiles;           // ceil(N / kTileKV)
    int launch;             // kLaunchPersistent | kLaunchGrid
    int decode;             // kDecodeDomain | kDecodeLinear
    int parts;              // interleaved subsets per head (domain decode; 1 for linear decode)
    int slots;              // workgroups per domain = grid / kDomains
    int chunks_per_domain;  // heads*parts / kDomains (domain decode)
    int rounds_per_chunk;   // persistent, domain decode: ceil(ceil(q_tiles/parts) / slots)
    int units_per_chunk;    // grid launch, domain decode: workgroups per chunk
    int tiles_per_wg;       // grid launch: consecutive tiles per workgroup (1 otherwise)
    int grid;               // workgroups launched (a multiple of kDomains)
    int local_iters;        // local iterations every workgroup runs through (some may be idle)
    int sync_heads;         // persistent, domain decode: the workgroups of a domain wait for each other between heads
    int sync_rounds;        // ... and after every round as well (a study of Sec. 3.4's lockstep; costs time)
    int qo_streaming;       // 1: O tiles leave through LDS as whole non-temporal lines; 2: Q tiles arrive that way; 3: both; 4: neither
};

struct Work {
    int head;        // b*H + h
    int tile;        // query tile index inside the head, -1: nothing to do in this iteration
    bool backward;   // walk the K/V tiles from the last visible one down to 0
    bool sync_after; // persistent domain decode: last round of a head that is not the domain's last
};


// max_slots in 1..resident_slots(d), tiles_per_wg in {1, 2}; the caller has validated them.
SAW_HD Schedule make_schedule(int heads, int N, bool causal, int launch, int decode, int max_slots, int tiles_per_wg,
                              int tile_q = kTileQ, bool align_rounds = false) {
    Schedule s;
    s.heads = heads;
    s.qo_streaming = 0;     // the caller's choice: not part of who computes what
    s.tile_q = tile_q;
    s.q_tiles = (N + tile_q - 1) / tile_q;
    s.kv_tiles = (N + kTileKV - 1) / kTileKV;
    s.launch = launch;
    s.decode = decode;
    s.tiles_per_wg = launch == kLaunchGrid ? tiles_per_wg : 1;
    s.parts = decode == kDecodeDomain ? kDomains / gcd_i(heads, kDomains) : 1;
    const int per_part = (s.q_tiles + s.parts - 1) / s.parts;     // tiles in the largest part
    s.chunks_per_domain = (int)(((long long)heads * s.parts) / kDomains);
    s.rounds_per_chunk = 0;
    s.units_per_chunk = 0;
    s.sync_heads = 0;
    s.sync_rounds = 0;
    const long long total = (long long)heads * s.q_tiles;
    if (launch == kLaunchPersistent) {
        if (decode == kDecodeDomain) {
            s.slots = per_part < max_slots ? per_part : max_slots;
            s.rounds_per_chunk = (per_part + s.slots - 1) / s.slots;
            s.local_iters = s.chunks_per_domain * s.rounds_per_chunk;
            // Waiting for the domain between heads pays only if its workgroups finish a head together:
            // every slot gets a tile in every round, and causal tiles pair up long with short.
            const bool even_load = s.q_tiles % (s.parts * s.slots) == 0 && (!causal || s.rounds_per_chunk % 2 == 0);
            s.sync_heads = even_load && s.chunks_per_domain > 1;
            s.sync_rounds = align_rounds && s.local_iters > 1;
        } else {
            const int want = ceil_div_i(total, kDomains);
            s.slots = want < max_slots ? want : max_slots;
            s.local_iters = ceil_div_i(total, (long long)kDomains * s.slots);
        }
    } else {
        if (decode == kDecodeDomain) {
            s.units_per_chunk = (per_part + s.tiles_per_wg - 1) / s.tiles_per_wg;
            s.slots = s.chunks_per_domain * s.units_per_chunk;
        } else {
            s.slots = ceil_div_i(ceil_div_i(total, s.tiles_per_wg), kDomains);
        }
        s.local_iters = s.tiles_per_wg;
    }
    s.grid = kDomains * s.slots;
    return s;
}

// What workgroup `wg` does in its local iteration `it` (0 <= it < local_iters).
SAW_HD Work decode_work(const Schedule& s, int wg, int it, bool causal, bool sawtooth) {
    Work w;
    w.head = 0;
    w.tile = -1;
    w.backward = false;
    w.sync_after = false;
    if (s.decode == kDecodeLinear) {
        // Alg. 2 / Alg. 3 as printed: one linear index over (head, tile), tile fastest.
        const long long k = s.launch == kLaunchPersistent ? (long long)wg + (long long)it * s.grid
                                                          : (long long)wg * s.tiles_per_wg + it;
        if (k < (long long)s.heads * s.q_tiles) {
            w.head = (int)(k / s.q_tiles);
            w.tile = (int)(k % s.q_tiles);
        }
        w.backward = sawtooth && (it & 1);
        return w;
    }
    const int domain = wg % kDomains, slot = wg / kDomains;
    int cs, u;
    if (s.launch == kLaunchPersistent) {
        cs = it / s.rounds_per_chunk;
        const int r = it - cs * s.rounds_per_chunk;
        u = r * s.slots + ((it & 1) ? s.slots - 1 - slot : slot);
        w.backward = sawtooth && (r & 1);
        w.sync_after = (s.sync_heads && r + 1 == s.rounds_per_chunk && cs + 1 < s.chunks_per_domain) ||
                       (s.sync_rounds && it + 1 < s.local_iters);
    } else {
        cs = slot / s.units_per_chunk;
        u = (slot - cs * s.units_per_chunk) * s.tiles_per_wg + it;
        w.backward = sawtooth && (it & 1);
    }
    const int c = cs * kDomains + domain;
    const int part = c % s.parts;
    w.head = c / s.parts;
    const int in_part = (s.q_tiles - part + s.parts - 1) / s.parts;
    if (u < in_part) w.tile = part + s.parts * (causal ? in_part - 1 - u : u);
    return w;
}

// K/V tiles visible to query tile t.
SAW_HD int visible_kv_tiles(const Schedule& s, int t, int N, bool causal) {
    if (!causal) return s.kv_tiles;
    long long last_row = (long long)(t + 1) * s.tile_q;
    if (last_row > N) last_row = N;
    return (int)((last_row + kTileKV - 1) / kTileKV);
}

}  // namespace sawattn
