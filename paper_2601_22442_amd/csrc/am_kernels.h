// Kernels of the AsyncMesh stage update (gfx950).  All of them are bound by HBM bandwidth; none is a
// contraction, so none uses the matrix cores.
#pragma once
#include "am_device.h"

namespace am {

// =============================================================================================
// Subset offsets:   k_subset_count (or k_subset_offsets)  ->  k_subset_scan
// =============================================================================================
// cnt[512] (LDS) holds the sizes of the tiles of superblock blockIdx.x: write their exclusive
// prefix to local_off and their total to sb_sum.  Called by all 256 threads after a barrier.
__device__ __forceinline__ void scan_superblock(const uint32_t *cnt, uint32_t *wave_tot, uint32_t ntiles,
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
    if (t_a < ntiles) local_off[t_a] = excl;
    if (t_a + 1 < ntiles) local_off[t_a + 1] = excl + a;
    if (threadIdx.x == 255) sb_sum[blockIdx.x] = base + incl;
}

// One workgroup (4 waves) per superblock of 512 tiles.  Pure integer hashing, no array reads.
// A tile's size is its number of selected coordinates (unit = 1: packed index lists) or that
// number rounded up to whole 128-byte lines of 32 floats (unit = 32: ring slots, where every tile
// owns whole lines).  Writes, per tile, the summed size of the tiles of the same superblock before
// it (local_off) and, per superblock, its total (sb_sum).
__global__ void __launch_bounds__(256)
k_subset_count(SubsetKey key, uint64_t n, uint32_t ntiles, uint32_t unit,
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
        if (lane == 0) cnt[k] = (total + unit - 1u) / unit;
    }
    __syncthreads();
    scan_superblock(cnt, wave_tot, ntiles, local_off, sb_sum);
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
    scan_superblock(cnt, wave_tot, ntiles, local_off, sb_sum);
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
enum : int { kOptSgdPlain = 0, kOptSgdMomentum = 1, kOptAdam = 2, kOptNone = 3 };   // kOptNone: w^ = w (averaging only)
enum : int { kFwdNone = 0, kFwdF32 = 1, kFwdBf16 = 2 };

struct StepArgs {
    float *w[kMaxReplicas];
    float *m[kMaxReplicas];
    float *v[kMaxReplicas];
    float *d[kMaxReplicas];
    void *fwd[kMaxReplicas];
    const void *g[kMaxReplicas];
    uint64_t n;
    uint32_t ntiles;
    uint32_t replicas;
    // averaging
    uint32_t do_send, do_recv, ema, same_slot;     // ema: a correction vector d is kept; same_slot: tau = 0,
                                                   // the average is of this step's w^
    uint32_t do_next;                              // also count the lines each tile will send next step
    uint32_t msg_dtype;                            // precision of the exchanged values: 0 fp32, 1 bf16, 2 E4M3
    SubsetKey key_send, key_recv, key_next;
    uint32_t *next_lines;                          // [ntiles], written when do_next
    float *ring_send;                              // slot written now: [replica][line][32]
    const float *ring_recv;                        // slot sent tau rounds ago
    const uint32_t *send_local_off, *send_sb_base; // first line of each tile = sb_base[tile >> 9] + local_off[tile]
    const uint32_t *recv_local_off, *recv_sb_base;
    uint32_t cap_lines;                            // lines (of 32 floats) per replica in a ring slot
    double coef_d, coef_s;                         // d <- coef_d d + coef_s (w^ - sent): EMA (1-lambda, lambda), eager (0, 1/R)
    // optimizer, every coefficient a per-step scalar evaluated once on the host in double:
    //   g  = grad_scale * g_raw                        (folded into b_m, b_v, c_g on the host)
    //   m' = a_m m + b_m g ;  v' = a_v v + b_v g^2
    //   w^ = w - (c_wd w + (c_g g + c_m m') / (c_v sqrt(v') + eps))           (Adam family)
    //   w^ = w - (c_wd w + c_m m')     resp.     w - (c_wd w + c_g g)          (SGD with / without momentum)
    // c_g, c_m, c_v hold the bias corrections and are per replica: replicas of unequal speed have made
    // unequal numbers of optimizer steps.  A replica whose bit in active_mask is clear makes no local
    // step in this launch (w^ = w; m, v kept; its gradient pointer is not read).
    double a_m, b_m, a_v, b_v, c_wd, eps;
    double c_g[kMaxReplicas], c_m[kMaxReplicas], c_v[kMaxReplicas];
    uint32_t active_mask;
    uint32_t lookahead;
    double gamma;
    const float *replica_scale;                    // NULL, or one more gradient factor per replica (DEVICE)
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
    F4 d;                   // EMA entries of the group (loaded only when its line receives)
};

// Local optimizer step on one group, from loaded operands.
template <int OPT>
__device__ __forceinline__ void local_step(const StepArgs &a, uint32_t i, const GroupIn &in,
                                           F4 &w_hat, F4 &m_new, F4 &v_new)
{
    // A replica that is idle in this tick goes through the same arithmetic with the coefficients of
    // the identity (m' = m, v' = v, w^ = w exactly); its gradient was not loaded.
    const bool idle = OPT != kOptNone && !((a.active_mask >> i) & 1u);
    const double rs = (OPT != kOptNone && a.replica_scale && !idle) ? (double)a.replica_scale[i] : 1.0;
    const double a_m = idle ? 1.0 : a.a_m, b_m = idle ? 0.0 : a.b_m;
    const double a_v = idle ? 1.0 : a.a_v, b_v = idle ? 0.0 : a.b_v;
    const double c_wd = idle ? 0.0 : a.c_wd;
    const double c_g = a.c_g[i], c_m = a.c_m[i], c_v = a.c_v[i];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (OPT == kOptNone) {                                 // averaging only: the caller's w is w^
            w_hat.v[j] = in.w.v[j];
            continue;
        }
        const double gj = rs * (double)in.g.v[j];              // grad_scale is folded into b_m, b_v, c_g
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

// Where the coordinates of one group sit in the subsets of this step.
struct GroupSubsets {
    uint32_t mask_send, mask_recv;      // bit j: coordinate 4*group + j is sent / received now
    uint32_t rank_send, rank_recv;      // rank of the first such coordinate among those of the tile
    uint32_t count_recv;                // received coordinates of the tile
    uint64_t run_send, run_recv;        // float offset, inside one replica's part of the slot, of the tile's lines
    uint32_t lines_send;                // whole lines the tile sends per replica
    bool line_recv;                     // the 128-byte line (of w, of d) holding the group receives something
};

// Issues the loads of replica i's dense operands for one group.
template <int OPT, bool GRAD_BF16>
__device__ __forceinline__ void load_group(const StepArgs &a, uint32_t i, uint64_t mu, int nvalid, GroupIn &in)
{
    in.w = load_f32x4(a.w[i], mu, nvalid);
    if ((a.active_mask >> i) & 1u)
        in.g = GRAD_BF16 ? load_bf16x4(static_cast<const uint16_t *>(a.g[i]), mu, nvalid)
                         : load_f32x4(static_cast<const float *>(a.g[i]), mu, nvalid);
    else
        in.g.v[0] = in.g.v[1] = in.g.v[2] = in.g.v[3] = 0.f;
    if (OPT != kOptSgdPlain) in.m = load_f32x4(a.m[i], mu, nvalid);
    if (OPT == kOptAdam) in.v = load_f32x4(a.v[i], mu, nvalid);
}

// What the averaging alone touches: the EMA entries of a line that receives, and (when there is no
// optimizer pass that reads w anyway) the weights of a group that sends or whose line receives.
template <int OPT>
__device__ __forceinline__ void load_group_sparse(const StepArgs &a, uint32_t i, uint64_t mu, int nvalid,
                                                  const GroupSubsets &s, GroupIn &in)
{
    if (a.ema && s.line_recv) in.d = load_f32x4(a.d[i], mu, nvalid);
    if (OPT == kOptNone && (s.mask_send != 0u || s.line_recv)) in.w = load_f32x4(a.w[i], mu, nvalid);
}

// Replica i of one group, from loaded operands to stored results.  sent_lds: what replica i sent
// tau rounds ago for the received coordinates of the tile, in rank order.
template <int OPT, int FWD>
__device__ __forceinline__ void step_replica(const StepArgs &a, uint32_t i, uint64_t mu, int nvalid, uint32_t lane,
                                             const GroupSubsets &s, const float (&abar)[4], GroupIn &in,
                                             const float *sent_lds, float *send_lds)
{
    F4 w_hat, m_new, v_new;
    local_step<OPT>(a, i, in, w_hat, m_new, v_new);

    if (s.lines_send) {
        // send: the tile's w^ values are gathered in LDS (the tail of the last line stays zero) and
        // leave as whole 128-byte lines
        uint32_t c = s.rank_send;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((s.mask_send >> j) & 1u) send_lds[c++] = w_hat.v[j];
        wave_lds_sync();
        float *__restrict__ dst = a.ring_send + (uint64_t)i * a.cap_lines * kLineFloats + s.run_send;
        for (uint32_t r = lane; r < s.lines_send * kLineFloats; r += 64u) __builtin_nontemporal_store(send_lds[r], dst + r);
        wave_lds_sync();
    }

    F4 w_new;
#pragma unroll
    for (int j = 0; j < 4; ++j) w_new.v[j] = w_hat.v[j];
    if (s.mask_recv) {                                     // receive: old average (+ EMA of staleness)
        uint32_t c = s.rank_recv;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((s.mask_recv >> j) & 1u) {
                if (a.ema) {
                    const float sent = a.same_slot ? w_hat.v[j] : sent_lds[c];
                    in.d.v[j] = (float)fma(a.coef_d, (double)in.d.v[j],
                                           a.coef_s * ((double)w_hat.v[j] - (double)sent));
                    w_new.v[j] = (float)((double)abar[j] + (double)in.d.v[j]);
                } else {
                    w_new.v[j] = abar[j];
                }
                ++c;
            }
    }
    if (a.ema && s.line_recv) store_f32x4(a.d[i], mu, nvalid, in.d);

    if (OPT == kOptNone) {                                 // averaging only: rewrite just the lines that receive
        if (s.line_recv) store_f32x4(a.w[i], mu, nvalid, w_new);
        return;
    }
    store_f32x4(a.w[i], mu, nvalid, w_new);
    if (OPT == kOptSgdMomentum || OPT == kOptAdam) store_f32x4(a.m[i], mu, nvalid, m_new);
    if (OPT == kOptAdam) store_f32x4(a.v[i], mu, nvalid, v_new);
    if (FWD != kFwdNone) {
        F4 f = w_new;
        if (a.lookahead) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                f.v[j] = (float)fma(a.gamma, (double)w_hat.v[j] - (double)in.w.v[j], (double)w_new.v[j]);
        }
        if (FWD == kFwdF32) store_f32x4(static_cast<float *>(a.fwd[i]), mu, nvalid, f);
        else store_bf16x4(static_cast<uint16_t *>(a.fwd[i]), mu, nvalid, f);
    }
}

// One workgroup per tile of 256 coordinates; its waves are the replicas (wave w takes replicas
// w, w + W, ...; W = min(R, 8) waves), one lane per group of 4 coordinates.  Each wave streams
// its replica's 1 KB of every array once and retires; measured on MI355X this shape, with
// non-temporal accesses, is the fastest way through the 4-read / 4-write stream mix of this update.
// Every wave hashes the tile's two subsets itself (integer work that hides under the memory time);
// the only thing the waves of a tile share is what the replicas sent tau rounds ago, which they
// put side by side in LDS to form the old average.
//
// This memory system writes 128-byte lines: a narrower write costs a read-modify-write of the line
// and, measured, several times the time of a whole-line write.  Both sparse structures are
// therefore laid out so that only whole lines are ever written:
//  * Ring slot: per replica, every tile owns ceil(count / 32) whole lines ([replica][line][32]);
//    a tile's selected values sit at the start of its lines in ascending coordinate order, the rest
//    of the last line is zero.  A wave gathers its values in LDS and stores whole lines.
//  * EMA vector d: dense in memory, touched only on received coordinates.  The 8 lanes that share
//    a 128-byte line of d load and store their groups together whenever any of them holds a
//    received coordinate, so the line is rewritten as a whole.
//
// FULL = every coordinate of the tile exists (all but possibly the last tile of the stage): all
// dense accesses are unconditional 128-bit ones.
template <int OPT, bool GRAD_BF16, int FWD, bool FULL>
__device__ __forceinline__ void step_tile(const StepArgs &a, uint32_t tile, uint32_t wave, uint32_t nwaves,
                                          uint32_t lane, float *sent_lds, float *send_lds)
{
    const uint32_t R = a.replicas;
    const uint64_t group = (uint64_t)tile * 64u + lane;
    const uint64_t mu = group * 4u;
    const int nvalid = FULL ? 4 : (mu >= a.n ? 0 : (a.n - mu >= 4u ? 4 : (int)(a.n - mu)));
    const uint64_t slot_floats = (uint64_t)a.cap_lines * kLineFloats;      // per replica

    // Averaging alone moves little per replica, so a wave keeps the loads of four of its replicas in
    // flight together; with the optimizer pass one replica's operands fill the registers.
    constexpr uint32_t DEPTH = OPT == kOptNone ? 4u : 1u;

    // first replica's dense operands go out before anything else waits on memory
    GroupIn in[DEPTH];
    if (OPT != kOptNone) load_group<OPT, GRAD_BF16>(a, wave, mu, nvalid, in[0]);

    // ---- subsets: which of my 4 coordinates are sent now / received now, and where the tile's
    //      lines start.  A tile whose lines would pass the slot capacity is left out, at send and at
    //      receive alike.
    GroupSubsets s;
    s.mask_send = s.mask_recv = s.rank_send = s.rank_recv = s.lines_send = s.count_recv = 0;
    s.run_send = s.run_recv = 0;
    if (a.do_send) {
        uint32_t count;
        s.mask_send = member_mask(a.key_send, group, nvalid);
        s.rank_send = wave_prefix_mask4(s.mask_send, count);
        const uint32_t first = a.send_sb_base[tile / kTilesPerSuperblock] + a.send_local_off[tile];
        s.lines_send = (count + kLineFloats - 1u) / kLineFloats;
        if ((uint64_t)first + s.lines_send > a.cap_lines) { s.mask_send = 0; s.lines_send = 0; count = 0; }
        s.run_send = (uint64_t)first * kLineFloats;
        if (a.same_slot) s.count_recv = count;
    }
    if (a.do_recv) {
        if (a.same_slot) {
            s.mask_recv = s.mask_send; s.rank_recv = s.rank_send; s.run_recv = s.run_send;
        } else {
            s.mask_recv = member_mask(a.key_recv, group, nvalid);
            s.rank_recv = wave_prefix_mask4(s.mask_recv, s.count_recv);
            const uint32_t first = a.recv_sb_base[tile / kTilesPerSuperblock] + a.recv_local_off[tile];
            const uint32_t lines = (s.count_recv + kLineFloats - 1u) / kLineFloats;
            if ((uint64_t)first + lines > a.cap_lines) { s.mask_recv = 0; s.count_recv = 0; }
            s.run_recv = (uint64_t)first * kLineFloats;
        }
    }
    {
        const uint64_t any = __ballot(s.mask_recv != 0u);
        s.line_recv = ((any >> (lane & ~7u)) & 0xFFull) != 0ull;
    }
#pragma unroll
    for (uint32_t k = 0; k < DEPTH; ++k)
        if (wave + k * nwaves < R) load_group_sparse<OPT>(a, wave + k * nwaves, mu, nvalid, s, in[k]);

    if (a.do_next && wave == 0) {                           // one wave per tile sizes the next step's send
        uint32_t count;
        (void)wave_prefix_mask4(member_mask(a.key_next, group, nvalid), count);
        if (lane == 0) a.next_lines[tile] = (count + kLineFloats - 1u) / kLineFloats;
    }

    if (s.lines_send) {                                     // zero the gather area once: line tails stay zero
        for (uint32_t r = lane; r < s.lines_send * kLineFloats; r += 64u) send_lds[r] = 0.f;
    }

    // ---- old average of the coordinates received now: every wave puts what its replicas sent
    //      (tau = 0: their w^ of this step) side by side in LDS, then each lane sums over the replicas
    float abar[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.do_recv) {                                        // same for the whole workgroup
        for (uint32_t i = wave; i < R; i += nwaves) {
            float *row = sent_lds + i * kTileCoords;
            if (a.same_slot) {
                if (s.count_recv) {
                    GroupIn pre;
                    F4 w_hat, m_new, v_new;
                    if (i == wave) {
                        pre = in[0];
                    } else {
                        if (OPT != kOptNone) load_group<OPT, GRAD_BF16>(a, i, mu, nvalid, pre);
                        load_group_sparse<OPT>(a, i, mu, nvalid, s, pre);
                    }
                    local_step<OPT>(a, i, pre, w_hat, m_new, v_new);
                    uint32_t c = s.rank_recv;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((s.mask_recv >> j) & 1u) row[c++] = w_hat.v[j];
                }
            } else {
                const float *__restrict__ src = a.ring_recv + (uint64_t)i * slot_floats + s.run_recv;
                for (uint32_t c = lane; c < s.count_recv; c += 64u) row[c] = src[c];
            }
        }
        __syncthreads();
        if (s.mask_recv) {
            const double inv_r = 1.0 / (double)R;
            uint32_t c = s.rank_recv;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((s.mask_recv >> j) & 1u) {
                    double sum = 0.;
                    for (uint32_t i = 0; i < R; ++i) sum += (double)quantize_message(sent_lds[i * kTileCoords + c], a.msg_dtype);
                    abar[j] = (float)(sum * inv_r);
                    ++c;
                }
        }
    }

    // ---- my replicas
    for (uint32_t base = wave; base < R; base += DEPTH * nwaves) {
        if (base != wave) {
#pragma unroll
            for (uint32_t k = 0; k < DEPTH; ++k) {
                const uint32_t i = base + k * nwaves;
                if (i < R) {
                    if (OPT != kOptNone) load_group<OPT, GRAD_BF16>(a, i, mu, nvalid, in[k]);
                    load_group_sparse<OPT>(a, i, mu, nvalid, s, in[k]);
                }
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < DEPTH; ++k) {
            const uint32_t i = base + k * nwaves;
            if (i < R) step_replica<OPT, FWD>(a, i, mu, nvalid, lane, s, abar, in[k], sent_lds + i * kTileCoords, send_lds);
        }
    }
}

// grid = one workgroup per tile; blockDim = 64 * min(R, 8); dynamic LDS = (R + waves) * 256 floats
template <int OPT, bool GRAD_BF16, int FWD>
__global__ void __launch_bounds__(512)
k_step(const StepArgs a)
{
    extern __shared__ float lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t tile = blockIdx.x;
    float *sent_lds = lds;                                              // [R][256]
    float *send_lds = lds + (a.replicas + wave) * kTileCoords;         // [wave][256]
    if ((uint64_t)(tile + 1u) * kTileCoords <= a.n)
        step_tile<OPT, GRAD_BF16, FWD, true>(a, tile, wave, nwaves, lane, sent_lds, send_lds);
    else
        step_tile<OPT, GRAD_BF16, FWD, false>(a, tile, wave, nwaves, lane, sent_lds, send_lds);
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
        F4 f;
#pragma unroll
        for (int j = 0; j < 4; ++j) f.v[j] = (float)fma(gamma, (double)a.v[j] - (double)b.v[j], (double)a.v[j]);
        if (OUT_BF16) store_bf16x4(static_cast<uint16_t *>(out), mu, nvalid, f);
        else store_f32x4(static_cast<float *>(out), mu, nvalid, f);
    }
}

// =============================================================================================
// Diagnostics: consensus error and variance of the EMA estimates over the replicas
// =============================================================================================
struct DiagArgs {
    const float *w[kMaxReplicas];
    const float *d[kMaxReplicas];      // all NULL when there is no correction vector
    uint64_t n;
    uint32_t replicas;
    uint32_t has_d;
};

// Workgroup b reduces the coordinates b, b + gridDim, ... (one coordinate per thread per pass) and
// writes its three partial results; a fixed grid and a fixed order make the result reproducible.
__global__ void __launch_bounds__(256)
k_diag_partial(const DiagArgs a, double *__restrict__ partial)
{
    __shared__ double red[3][256];
    double cons = 0., var_sum = 0., var_max = 0.;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    const double inv_r = 1.0 / (double)a.replicas;
    for (uint64_t mu = (uint64_t)blockIdx.x * 256u + threadIdx.x; mu < a.n; mu += stride) {
        double mean = 0.;
        for (uint32_t i = 0; i < a.replicas; ++i) mean += (double)a.w[i][mu];
        mean *= inv_r;
        for (uint32_t i = 0; i < a.replicas; ++i) { const double e = (double)a.w[i][mu] - mean; cons += e * e; }
        if (a.has_d) {
            double dm = 0., v = 0.;
            for (uint32_t i = 0; i < a.replicas; ++i) dm += (double)a.d[i][mu];
            dm *= inv_r;
            for (uint32_t i = 0; i < a.replicas; ++i) { const double e = (double)a.d[i][mu] - dm; v += e * e; }
            v *= inv_r;
            var_sum += v;
            var_max = v > var_max ? v : var_max;
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
