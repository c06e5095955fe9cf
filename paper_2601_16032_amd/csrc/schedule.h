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
//   * odd rounds hand the tiles out in reverse slot order, which evens out the causal cost
//     (tile i costs i+1 K/V tiles), and causal chunks start from their longest tile;
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

constexpr int kTileQ = 128;      // query rows per workgroup tile
constexpr int kTileKV = 64;      // key/value rows per streamed tile
constexpr int kThreads = 256;    // 4 wavefronts, 32 query rows each
constexpr int kDomains = 8;      // XCDs
constexpr int kMaxSlots = 64;    // 32 CUs per XCD x 2 resident workgroups per CU

struct Schedule {
    int heads;              // B*H
    int q_tiles;            // ceil(N / kTileQ)
    int kv_tiles;           // ceil(N / kTileKV)
    int parts;              // interleaved subsets per head
    int slots;              // workgroups per domain
    int chunks_per_domain;  // heads*parts / kDomains
    int rounds_per_chunk;   // ceil(ceil(q_tiles/parts) / slots)
};

SAW_HD int gcd_i(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

SAW_HD Schedule make_schedule(int heads, int N) {
    Schedule s;
    s.heads = heads;
    s.q_tiles = (N + kTileQ - 1) / kTileQ;
    s.kv_tiles = (N + kTileKV - 1) / kTileKV;
    s.parts = kDomains / gcd_i(heads, kDomains);
    int per_part = (s.q_tiles + s.parts - 1) / s.parts;     // tiles in the largest part
    s.slots = per_part < kMaxSlots ? per_part : kMaxSlots;
    s.chunks_per_domain = (int)(((long long)heads * s.parts) / kDomains);
    s.rounds_per_chunk = (per_part + s.slots - 1) / s.slots;
    return s;
}

// Tile taken by (domain, slot) in round `r` of the domain's `cs`-th chunk; -1 if it sits out.
SAW_HD int decode_tile(const Schedule& s, int domain, int slot, int cs, int r, bool causal, int* head) {
    int c = cs * kDomains + domain;
    int part = c % s.parts;
    *head = c / s.parts;
    int in_part = (s.q_tiles - part + s.parts - 1) / s.parts;
    int u = r * s.slots + ((r & 1) ? s.slots - 1 - slot : slot);
    if (u >= in_part) return -1;
    if (causal) u = in_part - 1 - u;
    return part + s.parts * u;
}

// K/V tiles visible to query tile t.
SAW_HD int visible_kv_tiles(const Schedule& s, int t, int N, bool causal) {
    if (!causal) return s.kv_tiles;
    long long last_row = (long long)(t + 1) * kTileQ;
    if (last_row > N) last_row = N;
    return (int)((last_row + kTileKV - 1) / kTileKV);
}

}  // namespace sawattn
