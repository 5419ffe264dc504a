// Kernels of the AsyncMesh stage update (gfx950).  All of them are bound by HBM bandwidth; none is a
// contraction, so none uses the matrix cores.
#pragma once
#include "am_device.h"

namespace am {

// =============================================================================================
// Subset offsets:   k_subset_count (or k_subset_offsets)  ->  k_subset_scan
// =============================================================================================
// cnt[512] (LDS) holds the sizes of the tiles of superblock blockIdx.x: write their exclusive
// prefix to local_off and their total to sb_sum.  pack: a tile's word also carries its own size in
// the high 8 bits (ring slots, where a tile owns at most 64 lines and a superblock at most 2^15).
// Called by all 256 threads after a barrier.
__device__ __forceinline__ void scan_superblock(const uint32_t *cnt, uint32_t *wave_tot, uint32_t ntiles, bool pack,
                                                uint32_t *__restrict__ local_off, uint32_t *__restrict__ sb_sum)
{
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t tile0 = blockIdx.x * kTilesPerSuperblock;
    // thread j owns entries 2j, 2j+1
    const uint32_t a = cnt[2 * threadIdx.x], b = cnt[2 * threadIdx.x + 1];
    uint32_t incl = a + b;                       // inclusive scan across the wave, by shuffles
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if ((int)lane >= off) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
    for (uint32_t w = 0; w < wave; ++w) base += wave_tot[w];
    const uint32_t excl = base + incl - (a + b);
    const uint32_t t_a = tile0 + 2 * threadIdx.x;
    if (t_a < ntiles) local_off[t_a] = pack ? (excl | (a << 24)) : excl;
    if (t_a + 1 < ntiles) local_off[t_a + 1] = pack ? ((excl + a) | (b << 24)) : excl + a;
    if (threadIdx.x == 255) sb_sum[blockIdx.x] = base + incl;
}

// One workgroup (4 waves) per superblock of 512 tiles.  Pure integer hashing, no array reads.
// A tile's size is ceil(count * mul / unit), count its number of selected coordinates:
// mul = unit = 1 for packed index lists; mul = replicas per block, unit = 32 for ring slots, where a
// tile owns whole 128-byte lines of [coordinate][replica] values.  Writes, per tile, the summed size
// of the tiles of the same superblock before it (local_off) and, per superblock, its total (sb_sum).
__global__ void __launch_bounds__(256)
k_subset_count(SubsetKey key, uint64_t n, uint32_t ntiles, uint32_t mul, uint32_t unit, uint32_t pack,
               uint32_t *__restrict__ local_off, uint32_t *__restrict__ sb_sum)
{
    __shared__ uint32_t cnt[kTilesPerSuperblock];
    __shared__ uint32_t wave_tot[4];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t tile0 = blockIdx.x * kTilesPerSuperblock;

    // wave w counts tiles tile0 + w, w+4, ... (adjacent waves hash adjacent tiles)
    for (uint32_t k = wave; k < kTilesPerSuperblock; k += 4) {
        const uint32_t tile = tile0 + k;
        uint32_t total = 0;
        if (tile < ntiles) {
            const uint64_t group = (uint64_t)tile * 64u + lane;
            const uint64_t mu = group * 4u;
            const int nvalid = mu >= n ? 0 : (n - mu >= 4u ? 4 : (int)(n - mu));
            (void)wave_prefix_mask4(member_mask(key, group, nvalid), total);
        }
        if (lane == 0) cnt[k] = (total * mul + unit - 1u) / unit;
    }
    __syncthreads();
    scan_superblock(cnt, wave_tot, ntiles, pack != 0u, local_off, sb_sum);
}

// Same, from tile sizes that are already in memory (the fused step kernel leaves the line counts
// of the next step's subset there, so that step needs no hashing pass of its own).
__global__ void __launch_bounds__(256)
k_subset_offsets(const uint32_t *__restrict__ tile_size, uint32_t ntiles,
                 uint32_t *__restrict__ local_off, uint32_t *__restrict__ sb_sum)
{
    __shared__ uint32_t cnt[kTilesPerSuperblock];
    __shared__ uint32_t wave_tot[4];
    const uint32_t tile0 = blockIdx.x * kTilesPerSuperblock;
    for (uint32_t k = threadIdx.x; k < kTilesPerSuperblock; k += 256u)
        cnt[k] = tile0 + k < ntiles ? tile_size[tile0 + k] : 0u;
    __syncthreads();
    scan_superblock(cnt, wave_tot, ntiles, true, local_off, sb_sum);
}

// Single workgroup: exclusive scan of the superblock totals, in place (sb[i] <- sum of sb[<i]),
// grand total to sb[nsb]; raises flag bit 0 when the total exceeds the ring slot capacity.
__global__ void __launch_bounds__(256)
k_subset_scan(uint32_t *__restrict__ sb, uint32_t nsb, uint32_t capacity, uint32_t *__restrict__ flags,
              uint64_t *__restrict__ count_out)
{
    __shared__ uint64_t part[256];
    const uint32_t per = (nsb + 255u) / 256u;
    const uint32_t lo = threadIdx.x * per;
    const uint32_t hi = lo + per < nsb ? lo + per : nsb;
    uint64_t s = 0;
    for (uint32_t i = lo; i < hi; ++i) s += sb[i];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t run = 0;
        for (int i = 0; i < 256; ++i) { const uint64_t x = part[i]; part[i] = run; run += x; }
        sb[nsb] = run > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)run;
        if (run > capacity && flags) atomicOr(flags, 1u);
        if (count_out) *count_out = run;
    }
    __syncthreads();
    uint64_t run = part[threadIdx.x];
    for (uint32_t i = lo; i < hi; ++i) { const uint32_t x = sb[i]; sb[i] = (uint32_t)run; run += x; }
}

// Ascending index list of a subset (for am_subset_indices).
__global__ void __launch_bounds__(256)
k_subset_write(SubsetKey key, uint64_t n, uint32_t ntiles, const uint32_t *__restrict__ local_off,
               const uint32_t *__restrict__ sb_base, uint64_t *__restrict__ out, uint64_t capacity)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t nwaves = gridDim.x * 4u;
    for (uint32_t tile = blockIdx.x * 4u + (threadIdx.x >> 6); tile < ntiles; tile += nwaves) {
        const uint64_t group = (uint64_t)tile * 64u + lane;
        const uint64_t mu = group * 4u;
        const int nvalid = mu >= n ? 0 : (n - mu >= 4u ? 4 : (int)(n - mu));
        const uint32_t mask = member_mask(key, group, nvalid);
        uint32_t total;
        uint64_t pos = (uint64_t)sb_base[tile / kTilesPerSuperblock] + local_off[tile] + wave_prefix_mask4(mask, total);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((mask >> j) & 1u) {
                if (pos < capacity) out[pos] = mu + j;
                ++pos;
            }
    }
}

// =============================================================================================
// Fused step kernel
// =============================================================================================
enum : int { kOptSgdPlain = 0, kOptSgdMomentum = 1, kOptAdam = 2 };
enum : int { kFwdNone = 0, kFwdF32 = 1, kFwdBf16 = 2 };

// What one replica's wave needs to know about its replica: 64 bytes, one scalar load.  The record
// of replica b rb + k sits in slot 8 b + k of StepArgs::rep, whatever rb is, so that a wave finds its
// record from its block and wave numbers alone, in the same breath as the kernel's other arguments.
// Slots of absent replicas (R not a multiple of rb) repeat the record of the block's first replica:
// their waves may load through it, and store nothing.
struct ReplicaArgs {
    float *w, *m, *v;
    void *fwd;
    const void *g;              // NULL: the replica makes no local step in this launch (w^ = w; m, v kept)
    // bias corrections of the optimizer, per replica: replicas of unequal speed have made unequal
    // numbers of optimizer steps
    double c_g, c_m, c_v;
};

struct StepArgs {
    uint64_t n;
    uint32_t ntiles;
    uint32_t replicas;
    // blocks: replicas b rb .. b rb + rb - 1 form block b; one wave of a workgroup per replica of a block
    uint32_t rb, rb_shift;                         // replicas per block (1, 2, 4 or 8) and its log2
    uint32_t nblocks;                              // ceil(replicas / rb)
    uint32_t blocks_per_wg;                        // 1 (grid = tiles x blocks), or nblocks when tau = 0 (grid = tiles)
    uint32_t lookahead;
    // averaging
    uint32_t do_send, do_recv, ema, same_slot;     // ema: a correction vector d is kept; same_slot: tau = 0,
                                                   // the average is of this step's w^
    uint32_t do_next;                              // also count the lines each tile will send next step
    uint32_t msg_dtype;                            // precision of the exchanged values: 0 fp32, 1 bf16, 2 E4M3
    uint32_t cap_lines;                            // lines (of 32 floats) per block in a ring slot
    const uint32_t *send_meta, *send_sb_base;      // tile's word: lines << 24 | offset in its superblock; first line = sb_base[tile >> 9] + offset
    const uint32_t *recv_meta, *recv_sb_base;
    float *ring_send;                              // slot written now: [block][line][32], a line = [coordinate][rb]
    const float *ring_recv;                        // slot sent tau rounds ago
    uint32_t *next_lines;                          // [ntiles], written when do_next
    const float *replica_scale;                    // NULL, or one more gradient factor per replica (DEVICE)
    SubsetKey key;                                 // seed, threshold and sampling rule; the step words are filled per job
    uint32_t step_lo[3], step_hi[3];               // the steps whose subsets are hashed: [0] received now, [1] sent now, [2] sent next step
    double coef_d, coef_s;                         // d <- coef_d d + coef_s (w^ - sent): EMA (1-lambda, lambda), eager (0, 1/R)
    // optimizer, every coefficient a per-step scalar evaluated once on the host in double:
    //   g  = grad_scale * g_raw                        (folded into b_m, b_v, c_g on the host)
    //   m' = a_m m + b_m g ;  v' = a_v v + b_v g^2
    //   w^ = w - (c_wd w + (c_g g + c_m m') / (c_v sqrt(v') + eps))           (Adam family)
    //   w^ = w - (c_wd w + c_m m')     resp.     w - (c_wd w + c_g g)          (SGD with / without momentum)
    double a_m, b_m, a_v, b_v, c_wd, eps;
    double gamma;
    float *d[kMaxReplicas];          // one array per replica, or (interleaved) one per block: [tiles * 256][rb]
    ReplicaArgs rep[kMaxReplicas];
};

// Precision.  State is fp32 in memory (the method's precision).  The accumulating expressions
// (moments, weight update, EMA, look-ahead) are evaluated in fp64 from the stored fp32 values
// and rounded once on store, so that rounding noise does not random-walk over hundreds of steps;
// on this chip an fp64 FMA issues at the rate of an unpacked fp32 FMA, and the kernel is bound by
// memory.  The square root and the quotient start from the fp32 hardware approximations and take
// one Newton step in fp64 each, which is far cheaper than fp64 sqrt / divide sequences.

// sqrt(x) of an fp32 value x >= 0, to (nearly) double accuracy
__device__ __forceinline__ double sqrt_refined(float x)
{
    if (x == 0.0f) return 0.0;
    const float s0 = sqrtf(x);
    const double s0d = (double)s0;
    const double residual = fma(-s0d, s0d, (double)x);                     // x - s0^2, exact to fp64
    return s0d + (double)((float)residual * (0.5f * __builtin_amdgcn_rcpf(s0)));
}

// num / den for den > 0, to (nearly) double accuracy
__device__ __forceinline__ double quotient_refined(double num, double den)
{
    const float rden = __builtin_amdgcn_rcpf((float)den);
    const float q0 = (float)num * rden;
    const double residual = fma(-(double)q0, den, num);                    // num - q0 den
    return (double)q0 + (double)((float)residual * rden);
}

// What one replica's update of one group reads from memory.
struct GroupIn {
    F4 w, g, m, v;          // weights, gradients (widened), moments
    F4 d;                   // EMA entries of the group (per-replica layout: loaded when its line receives)
};

// Local optimizer step on one group, from loaded operands.
template <int OPT>
__device__ __forceinline__ void local_step(const StepArgs &a, const ReplicaArgs &r, uint32_t i, const GroupIn &in,
                                           F4 &w_hat, F4 &m_new, F4 &v_new)
{
    // A replica that is idle in this tick goes through the same arithmetic with the coefficients of
    // the identity (m' = m, v' = v, w^ = w exactly); its gradient was not loaded.
    const bool idle = r.g == nullptr;
    const double rs = (a.replica_scale && !idle) ? (double)a.replica_scale[i] : 1.0;
    const double a_m = idle ? 1.0 : a.a_m, b_m = idle ? 0.0 : a.b_m;
    const double a_v = idle ? 1.0 : a.a_v, b_v = idle ? 0.0 : a.b_v;
    const double c_wd = idle ? 0.0 : a.c_wd;
    const double c_g = r.c_g, c_m = r.c_m, c_v = r.c_v;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double gj = idle ? 0.0 : rs * (double)in.g.v[j]; // grad_scale is folded into b_m, b_v, c_g; idle: what was loaded is not a gradient
        const double wo = (double)in.w.v[j];
        double step;                                           // what is subtracted besides the decay
        if (OPT == kOptSgdPlain) {
            step = c_g * gj;
        } else if (OPT == kOptSgdMomentum) {
            m_new.v[j] = (float)fma(a_m, (double)in.m.v[j], b_m * gj);
            step = c_m * (double)m_new.v[j];
        } else {
            m_new.v[j] = (float)fma(a_m, (double)in.m.v[j], b_m * gj);
            v_new.v[j] = (float)fma(a_v, (double)in.v.v[j], b_v * gj * gj);
            const double den = fma(c_v, sqrt_refined(v_new.v[j]), a.eps);
            const double num = fma(c_g, gj, c_m * (double)m_new.v[j]);
            step = quotient_refined(num, den);
        }
        w_hat.v[j] = (float)(wo - fma(c_wd, wo, idle ? 0.0 : step));
    }
}

// LDS written by some lanes of a wave is about to be read by other lanes of the same wave.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Where the coordinates of one group (= one lane) sit in the subsets of this step.
struct GroupSubsets {
    uint32_t mask_send, mask_recv;      // bit j: coordinate 4*group + j is sent / received now
    uint32_t rank_send, rank_recv;      // rank of the first such coordinate among those of the tile
    bool line_recv;                     // the 128-byte line of a per-replica array (8 lanes) holding the group receives something
    uint32_t d_slot;                    // interleaved d: float offset, in the LDS staging area, of the group's first entry
};

// LDS of one workgroup (floats): what the replicas sent tau rounds ago, the touched lines of d, the
// lines about to be sent, and the list of touched lines.
struct TileLds {
    float *recv;        // [nblocks][256 coordinates in rank order][rb]
    float *d;           // [touched line][32]         (interleaved d only)
    float *send;        // [256 coordinates in rank order][rb]
    uint32_t *list;     // [64] tile-local index of the q-th touched line of d
    uint8_t *masks;     // [0..63] the lanes' masks of the sent subset, [64..127] of the received one
    float *abar;        // [256] mean over the replicas of what they sent, per received coordinate in rank order
};

// Issues the loads of replica i's dense operands for one group.
template <int OPT, bool GRAD_BF16>
__device__ __forceinline__ void load_group(const ReplicaArgs &r, uint64_t tbase, uint32_t loff, int nvalid, GroupIn &in)
{
    in.w = load_f32x4(r.w + tbase, loff, nvalid);
    // An idle replica has no gradient: its wave reads its weights in their place (memory that is
    // surely there; the optimizer step drops the value), without a branch, so that no load waits
    // for another.
    const void *gp = r.g == nullptr ? static_cast<const void *>(r.w) : r.g;
    in.g = GRAD_BF16 ? load_bf16x4(static_cast<const uint16_t *>(gp) + tbase, loff, nvalid)
                     : load_f32x4(static_cast<const float *>(gp) + tbase, loff, nvalid);
    if (OPT != kOptSgdPlain) in.m = load_f32x4(r.m + tbase, loff, nvalid);
    if (OPT == kOptAdam) in.v = load_f32x4(r.v + tbase, loff, nvalid);
}

// What the averaging touches in the per-replica arrays besides the dense operands: the EMA entries of
// a line that receives (per-replica layout of d).
template <bool DIL>
__device__ __forceinline__ void load_group_sparse(const StepArgs &a, uint32_t i, uint64_t tbase, uint32_t loff, int nvalid,
                                                  const GroupSubsets &s, GroupIn &in)
{
    if (!DIL && a.ema && s.line_recv) in.d = load_f32x4(a.d[i] + tbase, loff, nvalid);
}

// Replica i (slot `slot` of its block) of one group, from loaded operands to stored results.
// recv_block: what the replicas of i's block sent tau rounds ago, [rank][rb].
template <int OPT, int FWD, bool DIL, bool TAU0>
__device__ __forceinline__ void step_replica(const StepArgs &a, const ReplicaArgs &r, uint32_t i, uint32_t slot, uint64_t tbase, uint32_t loff, int nvalid,
                                             const GroupSubsets &s, const bool tile_receives, const float (&abar)[4], GroupIn &in,
                                             F4 &w_hat, F4 &m_new, F4 &v_new, const float *recv_block, const TileLds &L)
{
    const uint32_t rb = a.rb;
    if (TAU0 || !DIL) local_step<OPT>(a, r, i, in, w_hat, m_new, v_new);      // (else: done by the caller while it waited)
    if (TAU0 || !DIL) {                                    // the moments are final: out they go, before the averaging needs registers
        if (OPT == kOptSgdMomentum || OPT == kOptAdam) store_f32x4(r.m + tbase, loff, nvalid, m_new);
        if (OPT == kOptAdam) store_f32x4(r.v + tbase, loff, nvalid, v_new);
    }

    if (s.mask_send) {                                     // send: into the staging lines, [rank][rb]
        uint32_t c = s.rank_send;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((s.mask_send >> j) & 1u) L.send[(c++) * rb + slot] = w_hat.v[j];
    }

    F4 w_new;
#pragma unroll
    for (int j = 0; j < 4; ++j) w_new.v[j] = w_hat.v[j];
    if (tile_receives) {                                   // receive: old average (+ EMA of staleness)
        // Same for the whole workgroup, and free of branches inside: every lane reads (a lane without
        // a received coordinate reads entry 0 and drops the result), so that the LDS reads of the four
        // coordinates are in flight together instead of one dependent round trip per coordinate.
        uint32_t cj[4], c = s.rank_recv;
#pragma unroll
        for (int j = 0; j < 4; ++j) { const uint32_t bit = (s.mask_recv >> j) & 1u; cj[j] = bit ? c : 0u; c += bit; }
        if (a.ema) {
            float sent[4], d_old[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t bit = (s.mask_recv >> j) & 1u;
                sent[j] = TAU0 ? w_hat.v[j] : recv_block[cj[j] * rb + slot];
                d_old[j] = DIL ? L.d[bit ? s.d_slot + (uint32_t)j * rb + slot : 0u] : in.d.v[j];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float d_new = (float)fma(a.coef_d, (double)d_old[j], a.coef_s * ((double)w_hat.v[j] - (double)sent[j]));
                if ((s.mask_recv >> j) & 1u) {
                    if (DIL) L.d[s.d_slot + (uint32_t)j * rb + slot] = d_new;
                    else in.d.v[j] = d_new;
                    w_new.v[j] = (float)((double)abar[j] + (double)d_new);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((s.mask_recv >> j) & 1u) w_new.v[j] = abar[j];
        }
    }
    if (!DIL && a.ema && s.line_recv) store_f32x4(a.d[i] + tbase, loff, nvalid, in.d);

    store_f32x4(r.w + tbase, loff, nvalid, w_new);
    if (FWD != kFwdNone) {
        // fwd = w + gamma (w^ - w_before): product and sum rounded separately in fp64, then ONE
        // rounding to the stored type
        double f[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            f[j] = a.lookahead ? __dadd_rn((double)w_new.v[j], __dmul_rn(a.gamma, (double)w_hat.v[j] - (double)in.w.v[j]))
                               : (double)w_new.v[j];
        if (FWD == kFwdF32) {
            F4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o.v[j] = (float)f[j];
            store_f32x4(static_cast<float *>(r.fwd) + tbase, loff, nvalid, o);
        } else {
            store_bf16x4_from_f64(static_cast<uint16_t *>(r.fwd) + tbase, loff, nvalid, f);
        }
    }
}

// Mean over the replicas, in replica order and in fp64, of what they sent for the coordinate of
// rank c of the tile (recv: [block][rank][RB]): the RB values of a block come with one or two wide
// LDS reads.
template <int RB>
__device__ __forceinline__ float replica_mean(const StepArgs &a, const float *recv, uint32_t c)
{
    double sum = 0.;
    for (uint32_t b = 0; b < a.nblocks; ++b) {
        const uint32_t nrep = a.replicas - b * RB;         // replicas present in this block (>= RB: all)
        const float *p = recv + b * (kTileCoords * RB) + c * RB;
        float x[RB];
        if (RB == 8) {
            const v4f lo = *reinterpret_cast<const v4f *>(p), hi = *reinterpret_cast<const v4f *>(p + 4);
            x[0] = lo.x; x[1 % RB] = lo.y; x[2 % RB] = lo.z; x[3 % RB] = lo.w;
            x[4 % RB] = hi.x; x[5 % RB] = hi.y; x[6 % RB] = hi.z; x[7 % RB] = hi.w;
        } else if (RB == 4) {
            const v4f lo = *reinterpret_cast<const v4f *>(p);
            x[0] = lo.x; x[1 % RB] = lo.y; x[2 % RB] = lo.z; x[3 % RB] = lo.w;
        } else if (RB == 2) {
            const v2f lo = *reinterpret_cast<const v2f *>(p);
            x[0] = lo.x; x[1 % RB] = lo.y;
        } else {
            x[0] = p[0];
        }
        if (a.msg_dtype != 0u) {
#pragma unroll
            for (int k = 0; k < RB; ++k) x[k] = quantize_message(x[k], a.msg_dtype);
        }
#pragma unroll
        for (int k = 0; k < RB; ++k)
            if ((uint32_t)k < nrep) sum += (double)x[k];
    }
    return (float)(sum * (1.0 / (double)a.replicas));
}

// One workgroup per (tile of 256 coordinates, block of rb <= 8 replicas); its rb waves are the
// replicas of the block, one lane per group of 4 coordinates.  Each wave streams its replica's 1 KB
// of every per-replica array once, with non-temporal accesses (measured on MI355X: the fastest way
// through the 4-read / 4-write stream mix of this update).
//
// This memory system moves 128-byte lines, and a partial write costs several whole ones.  S^t is
// the same for every replica, so the sparse structures keep the replicas of a block side by side,
// [coordinate][replica]: a line holds 32 / rb coordinates of all rb replicas and is written as a whole.
//  * Ring slot: per block, every tile owns ceil(count rb / 32) whole lines ([block][line][32]); the
//    selected values sit in ascending coordinate order, the rest of the last line is zero.  The
//    tile's word in the slot's offset table (a scalar load) says where its lines start and how
//    many there are, so the lines sent tau rounds ago are requested without any hashing, straight
//    into LDS; the waves gather this step's values in LDS and the lines leave with 16 bytes per thread.
//  * EMA vector d, interleaved layout: [coordinate][replica] per block.  Lines that hold a received
//    coordinate are copied to LDS (16 bytes per lane), updated there and written back whole.
//    Per-replica layout: dense per replica; the 8 lanes that share a 128-byte line of d load and
//    store their groups together whenever any of them holds a received coordinate.
// Hashing a subset costs ten rounds of two 32 x 32 -> 64 multiplies per lane; the subsets are the
// same for every wave of the workgroup, so (fused step) one wave hashes the received subset, one
// the sent one, one the next step's, and the others read the 4-bit masks from LDS after the barrier
// they have to pass anyway.  (Where the masks steer loads of per-replica arrays -- the per-replica
// layout of d -- every wave still hashes the received subset itself, so that those loads go out
// before the barrier.)
//
// FULL = every coordinate of the tile exists (all but possibly the last tile of the stage): all
// dense accesses are unconditional 128-bit ones.
// TAU0 = the average is of this very step's values (tau = 0): the workgroup walks all the blocks
// of its tile, because it needs every replica's new weights (a rarely used mode, kept out of the
// code of the common one).
template <int OPT, bool GRAD_BF16, int FWD, bool DIL, bool TAU0, bool FULL>
__device__ __forceinline__ void step_tile(const StepArgs &a, const uint32_t tile, const uint32_t b0, const uint32_t wave,
                                          const uint32_t lane, const TileLds &L)
{
    // One wave hashes the sent subset for all; so it is with the received subset, unless its masks steer
    // loads of per-replica arrays that should leave before the barrier (per-replica layout of d in the
    // fused step).
    constexpr bool kShareRecv = DIL;
    constexpr bool kShareSend = true;
    const uint32_t R = a.replicas, rb = a.rb, sh = a.rb_shift;
    const uint32_t flat = wave * 64u + lane;                               // 64 rb threads; thread f owns 16-byte chunk f
    const uint64_t group = (uint64_t)tile * 64u + lane;
    const uint64_t mu = group * 4u;
    const int nvalid = FULL ? 4 : (mu >= a.n ? 0 : (a.n - mu >= 4u ? 4 : (int)(a.n - mu)));
    // addresses in the per-replica arrays: a pointer that is the same for the whole wave plus a 32-bit lane offset
    const uint64_t tbase = (uint64_t)tile * kTileCoords;
    const uint32_t loff = lane * 4u;
    const uint64_t block_floats = (uint64_t)a.cap_lines * kLineFloats;     // one block's part of a ring slot
    const uint32_t tile_floats = kTileCoords * rb;                         // one tile's part of an interleaved array
    constexpr bool recv_is_send = TAU0;                                    // the host launches TAU0 iff do_recv && same_slot

    // ---- dense operands of my replica of the first block: nothing else is requested before them
    uint32_t i = b0 * rb + wave;
    ReplicaArgs rep = a.rep[8u * b0 + wave];               // my replica's pointers and coefficients, one scalar load
    GroupIn in;
    // (no condition on i < R: the record of an absent replica names the arrays of the block's first
    // replica, whose values its wave loads and never uses -- with a condition the compiler parks
    // the conversions of the loaded values, and with them a wait for memory, right behind the loads)
    load_group<OPT, GRAD_BF16>(rep, tbase, loff, nvalid, in);
    __builtin_amdgcn_sched_barrier(0);

    // ---- subsets: bit j of a lane's mask = coordinate 4 group + j is received / sent now.
    //      Jobs: 0 = the received subset, 1 = the sent one, 2 = the size of what the next step sends.
    //      A shared job is done by wave (job mod rb), the others by every wave for itself.
    GroupSubsets s;
    s.mask_send = s.mask_recv = s.rank_send = s.rank_recv = s.d_slot = 0;
    s.line_recv = false;
    const uint32_t lpl = 8u >> sh;                                         // lanes (groups) per 128-byte line of d
    const uint32_t leader = lane & ~(lpl - 1u);
    // interleaved d: the lines of the tile that hold a received coordinate go straight into LDS, requested
    // by the wave that hashes the received subset as soon as it knows them.  (Noting the touched lines
    // in memory when a subset is sent and reading them back before hashing was measured slower: the
    // scalar load of the note holds the hashing wave up for longer than the hashing takes.)
    auto request_d_lines = [&](const uint64_t leaders) {
        const uint32_t nlines = (uint32_t)__popcll(leaders);
        if (nlines) {
            if ((leaders >> lane) & 1ull) L.list[__popcll(leaders & ((1ull << lane) - 1ull))] = lane >> (3u - sh);
            wave_lds_sync();
            const float *src = a.d[b0] + (uint64_t)tile * tile_floats + (lane & 7u) * 4u;
            for (uint32_t q0 = 0; q0 < nlines; q0 += 8u) {
                const uint32_t q = q0 + (lane >> 3);
                if (q < nlines) lds_dma_16(src + L.list[q] * kLineFloats, L.d + q0 * kLineFloats);
            }
        }
    };
    auto lines_of = [&](const uint32_t mask) {              // bit = first lane of a line of d that holds a coordinate of the mask
        const uint64_t any = __ballot(mask != 0u);
        const bool touched = ((any >> leader) & ((1ull << lpl) - 1ull)) != 0ull;
        return (uint64_t)__ballot(touched && lane == leader);
    };
#pragma unroll
    for (uint32_t job = 0; job < 3u; ++job) {
        const bool shared = job == 0u ? kShareRecv : job == 1u ? kShareSend : true;
        if (shared && wave != (job & (rb - 1u))) continue;
        if (job == 0u && !a.do_recv) continue;
        if (job == 1u && (!a.do_send || recv_is_send)) continue;
        if (job == 2u && !(a.do_next && b0 == 0u)) continue;
        SubsetKey key = a.key;
        const uint32_t which = (job == 0u && recv_is_send) ? 1u : job;
        key.step_lo = a.step_lo[which]; key.step_hi = a.step_hi[which];
        const uint32_t mask = member_mask(key, group, nvalid);
        if (job == 0u) {
            s.mask_recv = mask;
            if (kShareRecv) L.masks[64u + lane] = (uint8_t)mask;
            if (DIL && a.ema && wave == 0u) request_d_lines(lines_of(mask));
        } else if (job == 1u) {
            s.mask_send = mask;
            if (kShareSend) L.masks[lane] = (uint8_t)mask;
        } else {
            uint32_t count;
            (void)wave_prefix_mask4(mask, count);
            if (lane == 0) a.next_lines[tile] = (count * rb + kLineFloats - 1u) / kLineFloats;
        }
    }
    // ---- the tile's words in the offset tables of the two slots (scalar loads)
    uint32_t word_s = 0, base_s = 0, word_r = 0, base_r = 0;
    if (a.do_send) { word_s = uniform_load(a.send_meta, tile); base_s = uniform_load(a.send_sb_base, tile / kTilesPerSuperblock); }
    if (a.do_recv && !TAU0) { word_r = uniform_load(a.recv_meta, tile); base_r = uniform_load(a.recv_sb_base, tile / kTilesPerSuperblock); }

    // ---- where the tile's lines sit in the two slots.  A tile whose lines would pass the slot
    //      capacity is left out, at send and at receive alike.
    uint32_t first_s = base_s + (word_s & 0xFFFFFFu), lines_s = word_s >> 24;
    uint32_t first_r = base_r + (word_r & 0xFFFFFFu), lines_r = word_r >> 24;
    bool keep_s = a.do_send != 0u, keep_r = a.do_recv != 0u;
    if ((uint64_t)first_s + lines_s > a.cap_lines) { keep_s = false; lines_s = 0; }
    if (recv_is_send) { first_r = first_s; lines_r = lines_s; keep_r = keep_s; }
    else if ((uint64_t)first_r + lines_r > a.cap_lines) { keep_r = false; lines_r = 0; }

    // ---- what every replica sent tau rounds ago: straight into LDS.  The chunks are dealt out from
    //      the last wave down: the first waves are busy hashing.
    const uint32_t wave_r = rb - 1u - wave;
    if (a.do_recv && !TAU0 && wave_r * 64u + lane < lines_r * 8u) {
        const float *src = a.ring_recv + (uint64_t)first_r * kLineFloats + (wave_r * 64u + lane) * 4u;
        for (uint32_t b = 0; b < a.nblocks; ++b)
            lds_dma_16(src + b * block_floats, L.recv + b * tile_floats + wave_r * 256u);
    }
    if (!keep_r) s.mask_recv = 0u;                          // (masks a wave hashed for itself)
    if (!keep_s) s.mask_send = 0u;

    // the masks of the hashing waves, ranks inside the tile, and where the group's d entries sit in LDS
    uint32_t count_recv = 0, d_lines = 0;
    auto finish_subsets = [&]() {
        if (kShareRecv) s.mask_recv = keep_r ? (uint32_t)L.masks[64u + lane] : 0u;
        if (kShareSend) s.mask_send = recv_is_send ? s.mask_recv : (keep_s ? (uint32_t)L.masks[lane] : 0u);
        uint32_t count_send;
        s.rank_send = wave_prefix_mask4(s.mask_send, count_send);
        if (recv_is_send) { s.rank_recv = s.rank_send; count_recv = count_send; }
        else s.rank_recv = wave_prefix_mask4(s.mask_recv, count_recv);
        const uint64_t any_recv = __ballot(s.mask_recv != 0u);
        s.line_recv = ((any_recv >> (lane & ~7u)) & 0xFFull) != 0ull;
        if (DIL && a.ema) {
            const bool touched = ((any_recv >> leader) & ((1ull << lpl) - 1ull)) != 0ull;
            const uint64_t leaders = __ballot(touched && lane == leader);
            d_lines = (uint32_t)__popcll(leaders);
            s.d_slot = (uint32_t)__popcll(leaders & ((1ull << leader) - 1ull)) * kLineFloats + (lane & (lpl - 1u)) * 4u * rb;
        }
    };

    if (!kShareRecv) {                                     // loads of per-replica arrays that the masks steer
        const uint64_t any_recv = __ballot(s.mask_recv != 0u);
        s.line_recv = ((any_recv >> (lane & ~7u)) & 0xFFull) != 0ull;
        if (i < R) load_group_sparse<DIL>(a, i, tbase, loff, nvalid, s, in);
    }

    // ---- staging lines of the send start at zero: line tails and the slots of absent replicas stay zero
    if (flat < lines_s * 8u) *reinterpret_cast<v4f *>(L.send + flat * 4u) = v4f{0.f, 0.f, 0.f, 0.f};

    // ---- tau = 0: the average is of this step's w^ : every wave puts those of its replicas in place
    if (recv_is_send) {
        if (kShareRecv) __syncthreads();                   // the masks are in LDS
        finish_subsets();
        if (count_recv) {
            for (uint32_t b = 0; b < a.nblocks; ++b) {
                const uint32_t ib = b * rb + wave;
                if (ib >= R) continue;
                GroupIn pre;
                F4 w_hat, m_new, v_new;
                if (b == b0) {
                    pre = in;
                } else {
                    load_group<OPT, GRAD_BF16>(a.rep[8u * b + wave], tbase, loff, nvalid, pre);
                    load_group_sparse<DIL>(a, ib, tbase, loff, nvalid, s, pre);
                }
                local_step<OPT>(a, a.rep[8u * b + wave], ib, pre, w_hat, m_new, v_new);
                uint32_t c = s.rank_recv;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if ((s.mask_recv >> j) & 1u) L.recv[b * tile_floats + (c++) * rb + wave] = w_hat.v[j];
            }
        }
    }
    // the local optimizer step needs nothing but the wave's own operands: it runs while the lines
    // for LDS and the other waves' operands are still on their way
    F4 w_hat, m_new, v_new;
    if (!TAU0 && DIL) local_step<OPT>(a, rep, i, in, w_hat, m_new, v_new);      // (per-replica d: its entries are in registers too)
    lds_dma_wait();
    __syncthreads();
    constexpr bool kEarlyLocal = !TAU0 && DIL;
    if (kEarlyLocal && i < R) {                            // the moments are final: out they go at once
        if (OPT == kOptSgdMomentum || OPT == kOptAdam) store_f32x4(rep.m + tbase, loff, nvalid, m_new);
        if (OPT == kOptAdam) store_f32x4(rep.v + tbase, loff, nvalid, v_new);
    }
    if (!recv_is_send) finish_subsets();

    // ---- old average of the coordinates received now: thread c forms the mean of the coordinate of
    //      rank c once for the whole workgroup (in fp64, in replica order); after one more barrier every
    //      lane picks up the means of its own coordinates (a lane with fewer than four reads entry 0 and
    //      drops it, so that the four reads are in flight together)
    float abar[4] = {0.f, 0.f, 0.f, 0.f};
    if (count_recv) {                                      // same for the whole workgroup
        for (uint32_t c = flat; c < count_recv; c += 64u * rb)
            L.abar[c] = rb == 8u ? replica_mean<8>(a, L.recv, c) : rb == 4u ? replica_mean<4>(a, L.recv, c)
                      : rb == 2u ? replica_mean<2>(a, L.recv, c) : replica_mean<1>(a, L.recv, c);
        __syncthreads();
        uint32_t c = s.rank_recv;
#pragma unroll
        for (int j = 0; j < 4; ++j) { const uint32_t bit = (s.mask_recv >> j) & 1u; abar[j] = L.abar[bit ? c : 0u]; c += bit; }
    }

    // my chunk of the touched lines of d: float offset inside the tile's part of the array
    const uint32_t d_chunk_off = (DIL && flat < d_lines * 8u) ? L.list[flat >> 3] * kLineFloats + (flat & 7u) * 4u : 0u;

    // ---- my replica of each block of this workgroup (one block, except when tau = 0 and R > 8)
    for (uint32_t bb = 0; bb < (TAU0 ? a.blocks_per_wg : 1u); ++bb) {
        const uint32_t b = b0 + bb;
        i = b * rb + wave;
        if (TAU0 && bb != 0u) {
            __syncthreads();                               // the staging areas are free again
            if (flat < lines_s * 8u) *reinterpret_cast<v4f *>(L.send + flat * 4u) = v4f{0.f, 0.f, 0.f, 0.f};
            if (DIL && flat < d_lines * 8u)
                lds_dma_16(a.d[b] + (uint64_t)tile * tile_floats + d_chunk_off, L.d + wave * 256u);
            if (i < R) {
                rep = a.rep[8u * b + wave];
                load_group<OPT, GRAD_BF16>(rep, tbase, loff, nvalid, in);
                load_group_sparse<DIL>(a, i, tbase, loff, nvalid, s, in);
            }
            lds_dma_wait();
            __syncthreads();
        }
        if (i < R) step_replica<OPT, FWD, DIL, TAU0>(a, rep, i, wave, tbase, loff, nvalid, s, count_recv != 0u, abar, in, w_hat, m_new, v_new, L.recv + b * tile_floats, L);
        __syncthreads();
        // whole lines leave with 16 bytes per thread
        if (flat < lines_s * 8u) {
            float *dst = a.ring_send + b * block_floats + (uint64_t)first_s * kLineFloats + flat * 4u;
            __builtin_nontemporal_store(*reinterpret_cast<const v4f *>(L.send + flat * 4u), reinterpret_cast<v4f *>(dst));
        }
        if (DIL && flat < d_lines * 8u) {
            float *dst = a.d[b] + (uint64_t)tile * tile_floats + d_chunk_off;
            __builtin_nontemporal_store(*reinterpret_cast<const v4f *>(L.d + flat * 4u), reinterpret_cast<v4f *>(dst));
        }
    }
}

// Floats of dynamic LDS a workgroup needs.
__host__ __device__ inline uint32_t step_lds_floats(uint32_t rb, uint32_t nblocks, bool d_interleaved)
{
    return nblocks * kTileCoords * rb + (d_interleaved ? kTileCoords * rb : 0u) + kTileCoords * rb + 64u + 32u + kTileCoords;
}

// grid = (tiles, blocks) (tau = 0: (tiles, 1)); blockDim = 64 rb; dynamic LDS = step_lds_floats() floats
// (at most 80 registers, so that three workgroups of eight waves fit a compute unit)
template <int OPT, bool GRAD_BF16, int FWD, bool DIL, bool TAU0>
__global__ void __launch_bounds__(512, 6)
k_step(const StepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t tile = blockIdx.x, b0 = TAU0 ? 0u : blockIdx.y;
    const uint32_t tile_floats = kTileCoords * a.rb;
    TileLds L;
    L.recv = lds;
    L.d = L.recv + a.nblocks * tile_floats;
    L.send = L.d + (DIL ? tile_floats : 0u);
    L.list = reinterpret_cast<uint32_t *>(L.send + tile_floats);
    L.masks = reinterpret_cast<uint8_t *>(L.list + 64);
    L.abar = reinterpret_cast<float *>(L.list + 96);
    if ((uint64_t)(tile + 1u) * kTileCoords <= a.n)
        step_tile<OPT, GRAD_BF16, FWD, DIL, TAU0, true>(a, tile, b0, wave, lane, L);
    else
        step_tile<OPT, GRAD_BF16, FWD, DIL, TAU0, false>(a, tile, b0, wave, lane, L);
}

// =============================================================================================
// Averaging alone (am_sparse_average): subset, send, replica mean, EMA correction and scatter
// (asynchronous sparse averaging equations) on weights the caller has already stepped.
//
// Only lines that hold a selected coordinate move, so the call lives on how many of those lines are
// in flight, not on bytes.  The fused kernel's shape (a wave per replica, staging in LDS, four
// barriers a tile) keeps four tiles per compute unit in flight; here ONE wave owns one (tile, block
// of replicas) and keeps the block's RB replicas side by side in registers: lane l holds the four
// coordinates of its group for every replica of the block.  The RB values of a coordinate are one
// aligned stretch of 4 RB bytes in the ring slot and in the interleaved EMA vector ([coordinate][RB]),
// so the lane reads and writes them with one or two 128-bit accesses: no LDS, no barrier, two dozen
// tiles per compute unit in flight.  (Several lanes write parts of one line within a few
// instructions of each other; these are ordinary cached stores, which the L2 merges.)
// Arithmetic and its order are those of the fused kernel: mean in fp64 in replica order, rounded to
// fp32; d <- coef_d d + coef_s (w^ - sent) and w = mean + d in fp64, rounded once each.
// =============================================================================================
template <int RB>
__device__ __forceinline__ void load_block_values(const float *p, float (&x)[RB])
{
    if constexpr (RB == 8) {
        const v4f lo = *reinterpret_cast<const v4f *>(p), hi = *reinterpret_cast<const v4f *>(p + 4);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w; x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    } else if constexpr (RB == 4) {
        const v4f lo = *reinterpret_cast<const v4f *>(p);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
    } else if constexpr (RB == 2) {
        const v2f lo = *reinterpret_cast<const v2f *>(p);
        x[0] = lo.x; x[1] = lo.y;
    } else {
        x[0] = p[0];
    }
}

template <int RB>
__device__ __forceinline__ void store_block_values(float *p, const float (&x)[RB])
{
    if constexpr (RB == 8) {
        *reinterpret_cast<v4f *>(p) = v4f{x[0], x[1], x[2], x[3]};
        *reinterpret_cast<v4f *>(p + 4) = v4f{x[4], x[5], x[6], x[7]};
    } else if constexpr (RB == 4) {
        *reinterpret_cast<v4f *>(p) = v4f{x[0], x[1], x[2], x[3]};
    } else if constexpr (RB == 2) {
        *reinterpret_cast<v2f *>(p) = v2f{x[0], x[1]};
    } else {
        p[0] = x[0];
    }
}

// The values block `b` of the replicas sends for the tile: the RB values of a selected coordinate side
// by side at the coordinate's rank; the rest of the tile's last line is zero.
template <int RB>
__device__ __forceinline__ void average_send_block(float *slot, const F4 (&w)[RB], uint32_t mask_send, uint32_t rank_send,
                                                   uint32_t count_send, uint32_t room, uint32_t lane)
{
    uint32_t c = rank_send;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (((mask_send >> j) & 1u) && c < room) {             // (the rank is below that by construction of the table)
            float x[RB];
#pragma unroll
            for (int k = 0; k < RB; ++k) x[k] = w[k].v[j];
            store_block_values<RB>(slot + (uint64_t)c * RB, x);
            ++c;
        }
    }
    if (count_send + lane < room) {                            // fewer than 32 / RB <= 32 lanes
        float x[RB];
#pragma unroll
        for (int k = 0; k < RB; ++k) x[k] = 0.f;
        store_block_values<RB>(slot + (uint64_t)(count_send + lane) * RB, x);
    }
}

// Coordinate j of the group receives the old average abar: EMA of the staleness of each replica of the
// block (own[k] = what replica k itself sent), corrected weight.  dp: the coordinate's RB entries of the
// interleaved EMA vector (DIL), else the entries are in dv.
template <bool DIL, int RB>
__device__ __forceinline__ void average_receive(const StepArgs &a, int j, float abar, const float (&own)[RB], float *dp,
                                                F4 (&w)[RB], F4 (&dv)[RB])
{
    if (a.ema) {
        float d_new[RB];
        if (DIL) {
            load_block_values<RB>(dp, d_new);
        } else {
#pragma unroll
            for (int k = 0; k < RB; ++k) d_new[k] = dv[k].v[j];
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            d_new[k] = (float)fma(a.coef_d, (double)d_new[k], a.coef_s * ((double)w[k].v[j] - (double)own[k]));
            w[k].v[j] = (float)((double)abar + (double)d_new[k]);
            if (!DIL) dv[k].v[j] = d_new[k];
        }
        if (DIL) store_block_values<RB>(dp, d_new);
    } else {
#pragma unroll
        for (int k = 0; k < RB; ++k) w[k].v[j] = abar;
    }
}

// grid = (ceil(tiles / 4), blocks) (TAU0: (ceil(tiles / 4), 1)); blockDim = 256: four waves, each with
// a tile of its own (no LDS).
// DIL: the EMA vectors are interleaved ([coordinate][RB] per block); else one flat array per replica.
// TAU0: the average is of this very call's values (tau = 0): the wave walks all blocks of its tile,
// once for the sums and the send, once more for the update (another wave must not rewrite a block's
// weights while this one still needs them for the mean).
template <bool DIL, int RB, bool TAU0>
__global__ void __launch_bounds__(256, (DIL && !TAU0) ? 6 : 4)     // at most 80 (else 128) registers: 24 (16) tiles per compute unit in flight
k_average(const StepArgs a)
{
    constexpr uint32_t kPerLine = kLineFloats / RB;                        // coordinates a ring line holds
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t tile = blockIdx.x * 4u + wave, b0 = TAU0 ? 0u : blockIdx.y;
    if (tile >= a.ntiles) return;
    const uint32_t R = a.replicas;
    const uint64_t group = (uint64_t)tile * 64u + lane;
    const uint64_t mu = group * 4u;
    const int nvalid = mu >= a.n ? 0 : (a.n - mu >= 4u ? 4 : (int)(a.n - mu));
    const uint64_t tbase = (uint64_t)tile * kTileCoords;
    const uint32_t loff = lane * 4u;
    const uint64_t block_floats = (uint64_t)a.cap_lines * kLineFloats;     // one block's part of a ring slot

    // ---- the subsets: bit j of a lane's mask = coordinate 4 group + j is received / sent now
    uint32_t mask_recv = 0, mask_send = 0;
    SubsetKey key = a.key;
    if (a.do_recv && !TAU0) {
        key.step_lo = a.step_lo[0]; key.step_hi = a.step_hi[0];
        mask_recv = member_mask(key, group, nvalid);
    }
    if (a.do_send) {
        key.step_lo = a.step_lo[1]; key.step_hi = a.step_hi[1];
        mask_send = member_mask(key, group, nvalid);
    }
    if (a.do_next && b0 == 0u) {                                           // how many lines the tile sends next step
        key.step_lo = a.step_lo[2]; key.step_hi = a.step_hi[2];
        uint32_t count;
        (void)wave_prefix_mask4(member_mask(key, group, nvalid), count);
        if (lane == 0) a.next_lines[tile] = (count * RB + kLineFloats - 1u) / kLineFloats;
    }

    // ---- where the tile's lines sit in the two slots; a tile whose lines would pass the slot
    //      capacity is left out, at send and at receive alike
    uint32_t word_s = 0, base_s = 0, word_r = 0, base_r = 0;
    if (a.do_send) { word_s = uniform_load(a.send_meta, tile); base_s = uniform_load(a.send_sb_base, tile / kTilesPerSuperblock); }
    if (a.do_recv && !TAU0) { word_r = uniform_load(a.recv_meta, tile); base_r = uniform_load(a.recv_sb_base, tile / kTilesPerSuperblock); }
    const uint32_t first_s = base_s + (word_s & 0xFFFFFFu), first_r = base_r + (word_r & 0xFFFFFFu);
    uint32_t lines_s = word_s >> 24, lines_r = word_r >> 24;
    if ((uint64_t)first_s + lines_s > a.cap_lines) { lines_s = 0; mask_send = 0u; }
    if ((uint64_t)first_r + lines_r > a.cap_lines) { lines_r = 0; mask_recv = 0u; }
    if (TAU0) mask_recv = mask_send;                                       // what is sent now is received now

    uint32_t count_send, count_recv;
    const uint32_t rank_send = wave_prefix_mask4(mask_send, count_send);
    const uint32_t rank_recv = TAU0 ? rank_send : wave_prefix_mask4(mask_recv, count_recv);
    if (TAU0) count_recv = count_send;
    const uint64_t any_recv = __ballot(mask_recv != 0u);
    const bool line_recv = ((any_recv >> (lane & ~7u)) & 0xFFull) != 0ull;    // my 128-byte line of a per-replica array receives
    const bool need_w = mask_send != 0u || line_recv;
    const double inv_replicas = 1.0 / (double)R;

    F4 w[RB], dv[RB];
    // the weights (and, per-replica layout, the EMA entries) of block b's replicas; an absent replica counts as zeros
    auto load_block = [&](const uint32_t b, const bool with_w, const bool with_d) {
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const uint32_t i = b * RB + k;
            if (with_w) {
#pragma unroll
                for (int j = 0; j < 4; ++j) w[k].v[j] = 0.f;
                if (i < R && need_w) w[k] = load_f32x4(a.rep[8u * b + k].w + tbase, loff, nvalid);
            }
            if (with_d) {
#pragma unroll
                for (int j = 0; j < 4; ++j) dv[k].v[j] = 0.f;
                if (!DIL && a.ema && i < R && line_recv) dv[k] = load_f32x4(a.d[i] + tbase, loff, nvalid);
            }
        }
    };
    // only lines that received are rewritten
    auto store_block = [&](const uint32_t b) {
        if (!line_recv) return;
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const uint32_t i = b * RB + k;
            if (i >= R) continue;
            store_f32x4(a.rep[8u * b + k].w + tbase, loff, nvalid, w[k]);
            if (!DIL && a.ema) store_f32x4(a.d[i] + tbase, loff, nvalid, dv[k]);
        }
    };

    if constexpr (!TAU0) {
        load_block(b0, true, true);
        if (a.do_send && lines_s != 0u)
            average_send_block<RB>(a.ring_send + b0 * block_floats + (uint64_t)first_s * kLineFloats, w, mask_send, rank_send,
                                   count_send, lines_s * kPerLine, lane);
        // ---- receive: old average of what every replica sent (+ EMA of staleness)
        if (count_recv != 0u) {                                            // same for the whole wave
            const float *slot = a.ring_recv + (uint64_t)first_r * kLineFloats;
            uint32_t c = rank_recv;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (((mask_recv >> j) & 1u) && c < lines_r * kPerLine) {   // (as at the send)
                    double sum = 0.;
                    float own[RB];
                    for (uint32_t b = 0; b < a.nblocks; ++b) {
                        float x[RB];
                        load_block_values<RB>(slot + b * block_floats + (uint64_t)c * RB, x);
                        const uint32_t nrep = R - b * RB;                  // replicas present in this block (>= RB: all)
#pragma unroll
                        for (int k = 0; k < RB; ++k) {
                            if (b == b0) own[k] = x[k];                    // my own staleness term takes the exact value
                            const float q = a.msg_dtype != 0u ? quantize_message(x[k], a.msg_dtype) : x[k];
                            if ((uint32_t)k < nrep) sum += (double)q;
                        }
                    }
                    average_receive<DIL, RB>(a, j, (float)(sum * inv_replicas), own,
                                             DIL ? a.d[b0] + (tbase + loff + (uint32_t)j) * RB : nullptr, w, dv);
                    ++c;
                }
            }
        }
        store_block(b0);
    } else {
        // ---- first walk: every block sends, and the sums over all replicas (in replica order) build up
        double sum[4] = {0., 0., 0., 0.};
        for (uint32_t b = 0; b < a.nblocks; ++b) {
            load_block(b, true, false);
            if (lines_s != 0u)
                average_send_block<RB>(a.ring_send + b * block_floats + (uint64_t)first_s * kLineFloats, w, mask_send, rank_send,
                                       count_send, lines_s * kPerLine, lane);
            const uint32_t nrep = R - b * RB;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!((mask_recv >> j) & 1u)) continue;
#pragma unroll
                for (int k = 0; k < RB; ++k) {
                    const float q = a.msg_dtype != 0u ? quantize_message(w[k].v[j], a.msg_dtype) : w[k].v[j];
                    if ((uint32_t)k < nrep) sum[j] += (double)q;
                }
            }
        }
        // ---- second walk: the update of every block (one block: its weights are still in registers)
        if (count_recv != 0u) {
            for (uint32_t b = 0; b < a.nblocks; ++b) {
                if (a.nblocks > 1u) load_block(b, true, false);
                load_block(b, false, true);
                uint32_t c = rank_recv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (((mask_recv >> j) & 1u) && c < lines_s * kPerLine) {
                        float own[RB];
#pragma unroll
                        for (int k = 0; k < RB; ++k) own[k] = w[k].v[j];   // no delay: what was sent is this very value
                        average_receive<DIL, RB>(a, j, (float)(sum[j] * inv_replicas), own,
                                                 DIL ? a.d[b] + (tbase + loff + (uint32_t)j) * RB : nullptr, w, dv);
                        ++c;
                    }
                }
                store_block(b);
            }
        }
    }
}

// =============================================================================================
// Stateless look-ahead: out = w + gamma (w - w_prev)
// =============================================================================================
template <bool OUT_BF16>
__global__ void __launch_bounds__(256)
k_lookahead(void *__restrict__ out, const float *__restrict__ w, const float *__restrict__ w_prev,
            uint64_t n, double gamma)
{
    const uint64_t ngroups = (n + 3u) / 4u;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t group = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; group < ngroups; group += stride) {
        const uint64_t mu = group * 4u;
        const int nvalid = n - mu >= 4u ? 4 : (int)(n - mu);
        const F4 a = load_f32x4(w, mu, nvalid), b = load_f32x4(w_prev, mu, nvalid);
        double f[4];                                   // product and sum rounded separately in fp64, then one rounding
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = __dadd_rn((double)a.v[j], __dmul_rn(gamma, (double)a.v[j] - (double)b.v[j]));
        if (OUT_BF16) {
            store_bf16x4_from_f64(static_cast<uint16_t *>(out), mu, nvalid, f);
        } else {
            F4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o.v[j] = (float)f[j];
            store_f32x4(static_cast<float *>(out), mu, nvalid, o);
        }
    }
}

// =============================================================================================
// Diagnostics: consensus error and variance of the EMA estimates over the replicas
// =============================================================================================
struct DiagArgs {
    const float *w[kMaxReplicas];
    const float *d[kMaxReplicas];      // d_stride == 1: one array per replica; else one per block of d_stride replicas,
                                       // [coordinate][d_stride] (padded to whole tiles); all NULL when there is no correction vector
    uint64_t n;
    uint32_t replicas;
    uint32_t has_d;
    uint32_t d_stride;                 // 1 (one array per replica) or the replicas per block (interleaved)
};

// The EMA entries of coordinates mu .. mu + 3 of every replica from the interleaved layout: per block
// the 4 RB values are contiguous (the arrays are padded to whole tiles, so all four coordinates exist).
template <int RMAX, int RB>
__device__ __forceinline__ void diag_load_interleaved(const DiagArgs &a, uint64_t mu, F4 (&x)[RMAX])
{
#pragma unroll
    for (int b = 0; b < RMAX / RB; ++b) {
        if ((uint32_t)(b * RB) >= a.replicas) continue;
        const v4f *p = reinterpret_cast<const v4f *>(a.d[b] + mu * RB);
        float t[4 * RB];
#pragma unroll
        for (int q = 0; q < RB; ++q) {
            const v4f u = __builtin_nontemporal_load(p + q);
            t[4 * q] = u.x; t[4 * q + 1] = u.y; t[4 * q + 2] = u.z; t[4 * q + 3] = u.w;
        }
#pragma unroll
        for (int k = 0; k < RB; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) x[b * RB + k].v[j] = t[j * RB + k];
    }
}

// Every thread takes groups of 4 coordinates (group = thread index, + threads of the grid, ...), holds
// the group's values of all replicas in registers (RMAX >= replicas of them, all requested before the
// first is used) and accumulates its three partial results; a fixed grid and a fixed order make the
// result reproducible.
template <int RMAX>
__global__ void __launch_bounds__(256)
k_diag_partial(const DiagArgs a, double *__restrict__ partial)
{
    __shared__ double red[3][256];
    double cons = 0., var_sum = 0., var_max = 0.;
    const uint32_t R = a.replicas;
    const uint64_t stride = (uint64_t)gridDim.x * 256u, ngroups = (a.n + 3u) / 4u;
    const double inv_r = 1.0 / (double)R;
    for (uint64_t g = (uint64_t)blockIdx.x * 256u + threadIdx.x; g < ngroups; g += stride) {
        const uint64_t mu = g * 4u;
        const int nvalid = a.n - mu >= 4u ? 4 : (int)(a.n - mu);
        F4 x[RMAX];
#pragma unroll
        for (int i = 0; i < RMAX; ++i)
            if ((uint32_t)i < R) x[i] = load_f32x4(a.w[i], mu, nvalid);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j >= nvalid) continue;
            double mean = 0.;
#pragma unroll
            for (int i = 0; i < RMAX; ++i) if ((uint32_t)i < R) mean += (double)x[i].v[j];
            mean *= inv_r;
#pragma unroll
            for (int i = 0; i < RMAX; ++i) if ((uint32_t)i < R) { const double e = (double)x[i].v[j] - mean; cons += e * e; }
        }
        if (a.has_d) {
#pragma unroll
            for (int i = 0; i < RMAX; ++i) {
                if ((uint32_t)i >= R) continue;
                if (a.d_stride == 1u) x[i] = load_f32x4(a.d[i], mu, nvalid);
            }
            if (a.d_stride == 8u) diag_load_interleaved<RMAX, 8>(a, mu, x);
            else if (a.d_stride == 4u) diag_load_interleaved<RMAX, 4>(a, mu, x);
            else if (a.d_stride == 2u) diag_load_interleaved<RMAX, 2>(a, mu, x);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (j >= nvalid) continue;
                double dm = 0., v = 0.;
#pragma unroll
                for (int i = 0; i < RMAX; ++i) if ((uint32_t)i < R) dm += (double)x[i].v[j];
                dm *= inv_r;
#pragma unroll
                for (int i = 0; i < RMAX; ++i) if ((uint32_t)i < R) { const double e = (double)x[i].v[j] - dm; v += e * e; }
                v *= inv_r;
                var_sum += v;
                var_max = v > var_max ? v : var_max;
            }
        }
    }
    red[0][threadIdx.x] = cons; red[1][threadIdx.x] = var_sum; red[2][threadIdx.x] = var_max;
    __syncthreads();
    for (uint32_t off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) {
            red[0][threadIdx.x] += red[0][threadIdx.x + off];
            red[1][threadIdx.x] += red[1][threadIdx.x + off];
            const double o = red[2][threadIdx.x + off];
            if (o > red[2][threadIdx.x]) red[2][threadIdx.x] = o;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partial[3 * blockIdx.x + 0] = red[0][0];
        partial[3 * blockIdx.x + 1] = red[1][0];
        partial[3 * blockIdx.x + 2] = red[2][0];
    }
}

__global__ void __launch_bounds__(256)
k_diag_final(const double *__restrict__ partial, uint32_t nblocks, uint64_t n, double *__restrict__ out3)
{
    __shared__ double red[3][256];
    double cons = 0., var_sum = 0., var_max = 0.;
    for (uint32_t b = threadIdx.x; b < nblocks; b += 256u) {
        cons += partial[3 * b]; var_sum += partial[3 * b + 1];
        const double o = partial[3 * b + 2];
        var_max = o > var_max ? o : var_max;
    }
    red[0][threadIdx.x] = cons; red[1][threadIdx.x] = var_sum; red[2][threadIdx.x] = var_max;
    __syncthreads();
    for (uint32_t off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) {
            red[0][threadIdx.x] += red[0][threadIdx.x + off];
            red[1][threadIdx.x] += red[1][threadIdx.x + off];
            const double o = red[2][threadIdx.x + off];
            if (o > red[2][threadIdx.x]) red[2][threadIdx.x] = o;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { out3[0] = red[0][0]; out3[1] = red[1][0] / (double)n; out3[2] = red[2][0]; }
}

// =============================================================================================
// Squared gradient norms (the stage's share of each replica's global norm, for clipping)
// =============================================================================================
struct NormArgs {
    const void *g[kMaxReplicas];
    uint64_t n;
    uint32_t replicas;
    uint32_t is_bf16;
};

// grid = (blocks, replicas); block (b, i) sums the squares of groups b, b + blocks, ... of replica i
__global__ void __launch_bounds__(256)
k_sqnorm_partial(const NormArgs a, double *__restrict__ partial)
{
    __shared__ double red[256];
    const uint32_t i = blockIdx.y;
    const uint64_t ngroups = (a.n + 3u) / 4u;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    double acc = 0.;
    for (uint64_t group = (uint64_t)blockIdx.x * 256u + threadIdx.x; group < ngroups; group += stride) {
        const uint64_t mu = group * 4u;
        const int nvalid = a.n - mu >= 4u ? 4 : (int)(a.n - mu);
        const F4 g = a.is_bf16 ? load_bf16x4(static_cast<const uint16_t *>(a.g[i]), mu, nvalid)
                               : load_f32x4(static_cast<const float *>(a.g[i]), mu, nvalid);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += (double)g.v[j] * (double)g.v[j];     // tail entries are 0
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (uint32_t off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[(uint64_t)i * gridDim.x + blockIdx.x] = red[0];
}

// one block per replica: fixed-order sum of its partials
__global__ void __launch_bounds__(256)
k_sqnorm_final(const double *__restrict__ partial, uint32_t nblocks, double *__restrict__ out)
{
    __shared__ double red[256];
    double acc = 0.;
    for (uint32_t b = threadIdx.x; b < nblocks; b += 256u) acc += partial[(uint64_t)blockIdx.x * nblocks + b];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (uint32_t off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = red[0];
}

}  // namespace am
