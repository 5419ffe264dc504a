// Host-side arithmetic of the AsyncMesh stage update that involves no device: subset threshold,
// replica blocks, ring slot capacity, workspace layout, and which ring slots a step sends to and
// receives from.  Plain C++ (no HIP), so that it can be compiled and tested on a machine without a GPU.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <cmath>

#include "../../include/asyncmesh.h"
#include "am_geometry.h"

namespace am_host {

inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// floor(p 2^32); 2^32 selects every coordinate (sampling model of the sparse-averaging lemma)
inline uint64_t subset_threshold(double p)
{
    if (!(p > 0.0)) return 0;
    if (p >= 1.0) return 1ull << 32;
    return (uint64_t)std::floor(p * 4294967296.0);
}

// B = round(1/p) of the stratified sampling variant
inline uint64_t stratified_block(double p)
{
    const long long B = std::llround(1.0 / p);
    return B < 1 ? 1 : (uint64_t)B;
}

// Replicas are cut into blocks of rb = min(8, R rounded up to a power of two) consecutive replicas;
// the sparse values of a block's replicas sit side by side in memory.
struct Blocks {
    uint32_t rb, rb_shift, nblocks;
};

inline Blocks block_geometry(uint32_t replicas)
{
    Blocks b{1, 0, 1};
    while (b.rb < replicas && b.rb < am::kMaxBlockReplicas) { b.rb <<= 1; ++b.rb_shift; }
    b.nblocks = (replicas + b.rb - 1) / b.rb;
    return b;
}

// Lines (of 32 floats) one block's part of a ring slot must hold.  Every tile of 256 coordinates
// owns ceil(X rb / 32) whole lines, X ~ Binomial(256, p) its number of selected coordinates; the
// slot has room for the expected total plus twelve standard deviations (and 64 lines).
//   by_line: aligned blocks of 32 coordinates are drawn as a whole (X = 32 Binomial(8, p))
//   strat_block != 0: stratified sampling with that block length (no chance involved)
inline uint64_t slot_capacity_lines(uint64_t ntiles, double p, uint32_t rb, bool by_line, uint64_t strat_block)
{
    const uint64_t lines_per_tile = am::kTileCoords * rb / am::kLineFloats;     // every coordinate selected
    const uint64_t all = ntiles * lines_per_tile;
    if (p >= 1.0) return all;
    if (strat_block) {     // a tile meets at most floor(255 / B) + 2 blocks, one member each
        const uint64_t members = std::min<uint64_t>(am::kTileCoords, (am::kTileCoords - 1) / strat_block + 2);
        return std::min(all, ntiles * ((members * rb + am::kLineFloats - 1) / am::kLineFloats));
    }
    double mean = 0.0, sq = 0.0;
    if (by_line) {         // Binomial(8, p) drawn lines of 32 coordinates, rb lines of values each
        const double per = am::kTileCoords / am::kLineFloats;
        mean = per * p * rb;
        sq = per * p * (1.0 - p) * rb * rb + mean * mean;
    } else {
        const double lp = std::log(p), lq = std::log1p(-p), T = am::kTileCoords;
        for (int k = 0; k <= (int)am::kTileCoords; ++k) {
            const double pmf = std::exp(std::lgamma(T + 1.0) - std::lgamma(k + 1.0) - std::lgamma(T - k + 1.0) + k * lp + (T - k) * lq);
            const double lines = (double)(((uint64_t)k * rb + am::kLineFloats - 1) / am::kLineFloats);
            mean += pmf * lines;
            sq += pmf * lines * lines;
        }
    }
    const double var = sq - mean * mean > 0.0 ? sq - mean * mean : 0.0;
    const double cap = std::ceil((double)ntiles * mean + 12.0 * std::sqrt((double)ntiles * var)) + 64.0;
    return cap >= (double)all ? all : (uint64_t)cap;
}

// workspace = [flags 256 B][reduction partials 32 x 1024 doubles][next_lines u32[ntiles]][meta x (slots + 1)][ring values x slots]
//   meta = tile words u32[ntiles] | sb_base u32[nsb + 1]      (the extra block serves am_subset_indices)
//   ring slot = nblocks * cap_lines * 32 fp32: [block][line][32], a line = [coordinate][replica in block]
struct Layout {
    uint32_t ntiles, nsb, slots;
    Blocks blocks;
    uint64_t cap_lines;
    uint64_t off_flags, off_reduce, off_next, off_meta, meta_stride, meta_sb_off, off_ring, ring_stride, total;
};

inline Layout make_layout(const am_config &c)
{
    Layout L{};
    L.ntiles = (uint32_t)((c.n + am::kTileCoords - 1) / am::kTileCoords);
    L.nsb = (L.ntiles + am::kTilesPerSuperblock - 1) / am::kTilesPerSuperblock;
    L.slots = c.delay + 1;
    L.blocks = block_geometry(c.replicas);
    const uint64_t all = (uint64_t)L.ntiles * (am::kTileCoords * L.blocks.rb / am::kLineFloats);
    L.cap_lines = c.ring_cap_lines ? std::min<uint64_t>(c.ring_cap_lines, all)
                                   : slot_capacity_lines(L.ntiles, c.fraction, L.blocks.rb, c.subset_granule == 32,
                                                         c.subset_kind == AM_SUBSET_STRATIFIED ? stratified_block(c.fraction) : 0);
    L.off_flags = 0;
    L.off_reduce = 256;
    L.off_next = L.off_reduce + (uint64_t)AM_MAX_REPLICAS * 1024 * 8;
    L.off_meta = L.off_next + round_up((uint64_t)L.ntiles * 4, 256);
    L.meta_sb_off = round_up((uint64_t)L.ntiles * 4, 256);
    L.meta_stride = L.meta_sb_off + round_up(((uint64_t)L.nsb + 1) * 4, 256);
    L.off_ring = L.off_meta + L.meta_stride * (L.slots + 1);
    L.ring_stride = round_up(L.cap_lines * am::kLineFloats * L.blocks.nblocks * 4, 256);
    L.total = L.off_ring + L.ring_stride * L.slots;
    return L;
}

// Floats of one array of the EMA vectors and how many arrays there are, per layout.
inline void d_layout_shape(const am_config &c, uint32_t *rb, uint32_t *arrays, uint64_t *floats)
{
    if (c.d_layout == AM_D_INTERLEAVED) {
        const Blocks b = block_geometry(c.replicas);
        *rb = b.rb; *arrays = b.nblocks;
        *floats = round_up(c.n, am::kTileCoords) * b.rb;
    } else {
        *rb = 1; *arrays = c.replicas; *floats = c.n;
    }
}

// What step t does to the ring: averaging happens at steps t with t mod K == 0 (round t / K); the
// round's values go to slot round mod (depth), depth = configured delay + 1; what was sent tau rounds
// ago (tau = the delay in force, <= the configured one) is received once t - tau K >= 1.
struct Round {
    bool send, recv, same_slot;
    uint32_t slot_send, slot_recv;
    uint64_t step_recv;
};

inline Round plan_round(uint64_t K, uint64_t depth, uint64_t tau, uint64_t t)
{
    Round r{};
    if (t % K != 0) return r;
    const uint64_t round = t / K;
    r.send = true;
    r.slot_send = (uint32_t)(round % depth);
    if (t >= tau * K + 1) {                       // s = t - tau K >= 1: something was sent that long ago
        r.recv = true;
        r.step_recv = t - tau * K;
        r.slot_recv = (uint32_t)((round - tau) % depth);
        r.same_slot = tau == 0;
    }
    return r;
}

}  // namespace am_host
