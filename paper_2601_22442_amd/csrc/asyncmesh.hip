// Host side of the C ABI declared in include/asyncmesh.h: argument checking, per-step scalars,
// workspace layout, ring bookkeeping and kernel launches.  No device work happens outside the
// kernels of am_kernels.h; nothing here allocates device memory.
#include "../../include/asyncmesh.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "am_host_logic.h"
#include "am_kernels.h"

#ifndef AM_SOURCE_HASH
#define AM_SOURCE_HASH "unknown"
#endif

// Scratch of am_subset_indices_static: per-tile offsets and per-superblock bases of one subset,
// for stages of up to kStaticMaxN coordinates.  Every GPU the library runs on holds its own copy of
// this array for the life of the process.  The name is a host-side stand-in: host code reaches the
// memory only through the address hipGetSymbolAddress returns for the current device.
namespace {
constexpr uint64_t kStaticMaxN = 1ull << 27;
constexpr uint32_t kStaticMaxTiles = (uint32_t)(kStaticMaxN / am::kTileCoords);
constexpr uint32_t kStaticMaxSb = kStaticMaxTiles / am::kTilesPerSuperblock;
}
static __device__ __align__(256) uint32_t scratch[kStaticMaxTiles + kStaticMaxSb + 64];

namespace {

using am_host::Layout;
using am_host::Round;

// message of the last failing call on this thread; a fixed buffer, so that reporting an error
// allocates nothing and cannot throw
thread_local char g_last_error[512] = "";

am_status fail(am_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

#define AM_HIP(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) return fail(AM_EHIP, "%s: %s", #call, hipGetErrorString(e_));   \
    } while (0)

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t *g_scratch_ptr[kMaxDevices] = {};

// Device address of the static scratch array on the CURRENT device, looked up once per device.
am_status resolve_static_scratch(int device, uint32_t **out)
{
    if (device < 0 || device >= kMaxDevices) return fail(AM_EINVAL, "device %d is beyond the %d the static scratch table covers", device, kMaxDevices);
    try {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[device]) {
            void *p = nullptr;
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return fail(AM_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
            g_scratch_ptr[device] = static_cast<uint32_t *>(p);
        }
        *out = g_scratch_ptr[device];
    } catch (...) {
        return fail(AM_EHIP, "could not lock the static scratch table");
    }
    return AM_OK;
}

am_status check_config(const am_config *c)
{
    if (!c) return fail(AM_EINVAL, "config is NULL");
    if (c->n == 0 || c->n >= (1ull << 32) - (1ull << 20)) return fail(AM_EINVAL, "n=%llu out of range [1, 2^32-2^20)", (unsigned long long)c->n);
    if (c->replicas == 0 || c->replicas > AM_MAX_REPLICAS) return fail(AM_EINVAL, "replicas=%u out of range [1, %u]", c->replicas, AM_MAX_REPLICAS);
    if (c->avg_interval == 0) return fail(AM_EINVAL, "avg_interval must be >= 1");
    if (c->delay > 4096) return fail(AM_EINVAL, "delay=%u is larger than 4096 rounds", c->delay);
    if (!(c->fraction > 0.0) || !(c->fraction <= 1.0)) return fail(AM_EINVAL, "fraction=%g not in (0, 1]", c->fraction);
    if (c->optimizer > AM_OPT_NADAMW) return fail(AM_EINVAL, "unknown optimizer %u", c->optimizer);
    if (c->correction > AM_CORR_EAGER) return fail(AM_EINVAL, "unknown correction %u", c->correction);
    if (c->fwd_dtype > AM_BF16 || c->grad_dtype > AM_BF16) return fail(AM_EINVAL, "unknown dtype");
    if (c->msg_dtype > AM_MSG_E4M3) return fail(AM_EINVAL, "unknown msg_dtype %u", c->msg_dtype);
    if (c->subset_granule != 0 && c->subset_granule != 1 && c->subset_granule != 32) return fail(AM_EINVAL, "subset_granule=%u is not 1 or 32", c->subset_granule);
    if (c->subset_kind > AM_SUBSET_STRATIFIED) return fail(AM_EINVAL, "unknown subset_kind %u", c->subset_kind);
    if (c->subset_kind == AM_SUBSET_STRATIFIED && c->subset_granule == 32) return fail(AM_EINVAL, "the stratified subset has no line-granular form (subset_granule must be 1)");
    if (c->subset_kind == AM_SUBSET_STRATIFIED && am_host::stratified_block(c->fraction) > (1ull << 31)) return fail(AM_EINVAL, "fraction=%g gives a block longer than 2^31", c->fraction);
    if (c->d_layout > AM_D_INTERLEAVED) return fail(AM_EINVAL, "unknown d_layout %u", c->d_layout);
    if (!(c->beta1 >= 0.f && c->beta1 < 1.f)) return fail(AM_EINVAL, "beta1=%g not in [0, 1)", c->beta1);
    if (c->optimizer != AM_OPT_SGD && !(c->beta2 >= 0.f && c->beta2 < 1.f)) return fail(AM_EINVAL, "beta2=%g not in [0, 1)", c->beta2);
    if (c->optimizer != AM_OPT_SGD && !(c->eps >= 0.f)) return fail(AM_EINVAL, "eps=%g negative", c->eps);
    if (!std::isfinite(c->weight_decay) || !std::isfinite(c->gamma)) return fail(AM_EINVAL, "weight_decay / gamma not finite");
    return AM_OK;
}

}  // namespace

constexpr uint32_t kMaxProfiledLaunches = 4096;

struct am_state {
    am_config cfg;
    Layout lay;
    hipStream_t stream;
    int device;
    uint32_t grid_sparse;
    float *w[AM_MAX_REPLICAS], *m[AM_MAX_REPLICAS], *v[AM_MAX_REPLICAS];
    float *d[AM_MAX_REPLICAS];   // per replica, or (interleaved layout) per block
    uint32_t d_arrays, d_rb;     // how many entries of d are in use; replicas per array (1 = per replica)
    uint64_t d_floats;           // floats per array of d
    void *fwd[AM_MAX_REPLICAS];
    bool has_fwd;
    char *ws;
    uint64_t last_t;
    uint64_t next_lines_step;    // the step whose send subset next_lines() was sized for (0 = none)
    uint32_t delay_now;          // the delay in force (<= cfg.delay, which sizes the ring)
    bool overflow_seen;          // am_read_flags has reported a subset that did not fit its ring slot
    // per replica, because replicas of unequal speed make unequal numbers of local steps:
    uint64_t opt_steps[AM_MAX_REPLICAS];     // optimizer steps made so far (the t of the bias corrections)
    double mu_product[AM_MAX_REPLICAS];      // NAdam: running product of the momentum schedule
    uint64_t threshold;
    uint32_t *static_scratch;    // this device's copy of the static scratch array (am_subset_indices_static)
    // profiling of the fused kernel: a fixed pool of event pairs, created on first use
    bool profiling;
    hipEvent_t ev_pool[2 * kMaxProfiledLaunches];
    uint32_t ev_created, ev_used;

    uint32_t *flags() const { return reinterpret_cast<uint32_t *>(ws + lay.off_flags); }
    double *reduce_partials() const { return reinterpret_cast<double *>(ws + lay.off_reduce); }
    uint32_t *next_lines() const { return reinterpret_cast<uint32_t *>(ws + lay.off_next); }
    uint32_t *meta_local(uint32_t slot) const { return reinterpret_cast<uint32_t *>(ws + lay.off_meta + lay.meta_stride * slot); }
    uint32_t *meta_sb(uint32_t slot) const { return reinterpret_cast<uint32_t *>(ws + lay.off_meta + lay.meta_stride * slot + lay.meta_sb_off); }
    float *ring(uint32_t slot) const { return reinterpret_cast<float *>(ws + lay.off_ring + lay.ring_stride * slot); }
};

namespace {

am::SubsetKey make_key(const am_state *st, uint64_t step)
{
    am::SubsetKey k;
    k.seed_lo = (uint32_t)st->cfg.seed;
    k.seed_hi = (uint32_t)(st->cfg.seed >> 32);
    k.step_lo = (uint32_t)step;
    k.step_hi = (uint32_t)(step >> 32);
    k.threshold = st->threshold;
    k.mode = st->cfg.subset_kind == AM_SUBSET_STRATIFIED ? am::kDrawStratified
           : st->cfg.subset_granule == 32 ? am::kDrawLine : am::kDrawCoordinate;
    k.block = st->cfg.subset_kind == AM_SUBSET_STRATIFIED ? (uint32_t)am_host::stratified_block(st->cfg.fraction) : 0u;
    return k;
}

// Offsets of S^step in ring slot `slot`: per tile, the lines it owns and where they start in its
// superblock; per superblock, where it starts in the slot.
am_status launch_ring_offsets(am_state *st, uint64_t step, uint32_t slot)
{
    const Layout &L = st->lay;
    if (st->next_lines_step == step && step != 0) {
        // the previous fused step already sized this subset's tiles
        am::k_subset_offsets<<<L.nsb, 256, 0, st->stream>>>(st->next_lines(), L.ntiles, st->meta_local(slot), st->meta_sb(slot));
    } else {
        am::k_subset_count<<<L.nsb, 256, 0, st->stream>>>(make_key(st, step), st->cfg.n, L.ntiles, L.blocks.rb, am::kLineFloats, 1u,
                                                          st->meta_local(slot), st->meta_sb(slot));
    }
    AM_HIP(hipGetLastError());
    const uint32_t cap = L.cap_lines > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)L.cap_lines;
    am::k_subset_scan<<<1, 256, 0, st->stream>>>(st->meta_sb(slot), L.nsb, cap, st->flags(), nullptr);
    AM_HIP(hipGetLastError());
    return AM_OK;
}

am_status check_index_list_args(const am_state *st, const uint64_t *dev_out, uint64_t capacity, const uint64_t *dev_count)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (!dev_count) return fail(AM_EINVAL, "dev_count is NULL");
    if (!dev_out && capacity) return fail(AM_EINVAL, "dev_out is NULL with capacity > 0");
    if (!aligned(dev_out, 8) || !aligned(dev_count, 8)) return fail(AM_EALIGN, "pointer not 8-byte aligned");
    return AM_OK;
}

// S^t as an ascending index list: sizes of the tiles (in coordinates) -> offsets -> indices.  local_off
// (ntiles words) and sb_base (nsb + 1 words) are the scratch the three kernels share; every word of
// them that is read is written first, so the scratch needs no clearing.
am_status launch_index_list(am_state *st, uint64_t t, uint32_t *local_off, uint32_t *sb_base,
                            uint64_t *dev_out, uint64_t capacity, uint64_t *dev_count)
{
    const Layout &L = st->lay;
    am::k_subset_count<<<L.nsb, 256, 0, st->stream>>>(make_key(st, t), st->cfg.n, L.ntiles, 1u, 1u, 0u, local_off, sb_base);
    AM_HIP(hipGetLastError());
    am::k_subset_scan<<<1, 256, 0, st->stream>>>(sb_base, L.nsb, 0u, nullptr, dev_count);
    AM_HIP(hipGetLastError());
    if (capacity) {
        am::k_subset_write<<<st->grid_sparse, 256, 0, st->stream>>>(make_key(st, t), st->cfg.n, L.ntiles, local_off, sb_base, dev_out, capacity);
        AM_HIP(hipGetLastError());
    }
    return AM_OK;
}

Round plan_round(const am_state *st, uint64_t t)
{
    return am_host::plan_round(st->cfg.avg_interval, (uint64_t)st->cfg.delay + 1, st->delay_now, t);
}

// One workgroup per (tile, block of replicas), one wave per replica of the block; when the average
// is of this very step's values (tau = 0) a workgroup walks all the blocks of its tile, because it
// needs every replica's new weights.
template <int OPT, bool GBF, int FWD, bool DIL>
am_status launch_step_tau(am_state *st, const am::StepArgs &a)
{
    const am_host::Blocks &B = st->lay.blocks;
    const bool tau0 = a.do_recv && a.same_slot;
    const dim3 grid(st->lay.ntiles, tau0 ? 1u : B.nblocks), block(64u * B.rb);
    const size_t lds = (size_t)am::step_lds_floats(B.rb, B.nblocks, DIL) * sizeof(float);
    if (tau0) am::k_step<OPT, GBF, FWD, DIL, true><<<grid, block, lds, st->stream>>>(a);
    else am::k_step<OPT, GBF, FWD, DIL, false><<<grid, block, lds, st->stream>>>(a);
    AM_HIP(hipGetLastError());
    return AM_OK;
}

template <int OPT, bool GBF, int FWD>
am_status launch_step_layout(am_state *st, const am::StepArgs &a)
{
    if (st->cfg.d_layout == AM_D_INTERLEAVED && a.ema) return launch_step_tau<OPT, GBF, FWD, true>(st, a);
    return launch_step_tau<OPT, GBF, FWD, false>(st, a);
}

template <int OPT, bool GBF>
am_status launch_step_fwd(am_state *st, const am::StepArgs &a)
{
    if (!st->has_fwd) return launch_step_layout<OPT, GBF, am::kFwdNone>(st, a);
    if (st->cfg.fwd_dtype == AM_F32) return launch_step_layout<OPT, GBF, am::kFwdF32>(st, a);
    return launch_step_layout<OPT, GBF, am::kFwdBf16>(st, a);
}

template <int OPT>
am_status launch_step_grad(am_state *st, const am::StepArgs &a)
{
    return st->cfg.grad_dtype == AM_BF16 ? launch_step_fwd<OPT, true>(st, a) : launch_step_fwd<OPT, false>(st, a);
}

// The averaging-only kernel: one wave per (tile, block of replicas); with tau = 0 (the average is of this
// call's own values) one wave per tile, which walks the blocks.
template <bool DIL, bool TAU0>
am_status launch_average(am_state *st, const am::StepArgs &a)
{
    const am_host::Blocks &B = st->lay.blocks;
    const dim3 grid((st->lay.ntiles + 3u) / 4u, TAU0 ? 1u : B.nblocks), block(256);
    switch (B.rb) {
    case 8: am::k_average<DIL, 8, TAU0><<<grid, block, 0, st->stream>>>(a); break;
    case 4: am::k_average<DIL, 4, TAU0><<<grid, block, 0, st->stream>>>(a); break;
    case 2: am::k_average<DIL, 2, TAU0><<<grid, block, 0, st->stream>>>(a); break;
    default: am::k_average<DIL, 1, TAU0><<<grid, block, 0, st->stream>>>(a); break;
    }
    AM_HIP(hipGetLastError());
    return AM_OK;
}

// The averaging part of the kernel arguments for step t; launches the offsets pass when t sends.
am_status fill_averaging(am_state *st, uint64_t t, float lambda_t, const Round &r, am::StepArgs &a)
{
    const am_config &c = st->cfg;
    const am_host::Blocks &B = st->lay.blocks;
    a.n = c.n; a.ntiles = st->lay.ntiles; a.replicas = c.replicas;
    a.rb = B.rb; a.rb_shift = B.rb_shift; a.nblocks = B.nblocks;
    a.blocks_per_wg = (r.recv && r.same_slot) ? B.nblocks : 1u;
    a.cap_lines = st->lay.cap_lines > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)st->lay.cap_lines;
    a.ema = c.correction != AM_CORR_NONE;
    a.msg_dtype = c.msg_dtype;
    if (c.correction == AM_CORR_EAGER) { a.coef_d = 0.0; a.coef_s = 1.0 / (double)c.replicas; }
    else { a.coef_d = 1.0 - (double)lambda_t; a.coef_s = (double)lambda_t; }
    a.do_send = r.send; a.do_recv = r.recv; a.same_slot = r.same_slot;
    a.key = make_key(st, 0);
    for (uint32_t k = 0; k < st->d_arrays; ++k) a.d[k] = st->d[k];
    if (r.send) {
        if (am_status s = launch_ring_offsets(st, t, r.slot_send)) return s;
        a.step_lo[1] = (uint32_t)t; a.step_hi[1] = (uint32_t)(t >> 32);
        a.ring_send = st->ring(r.slot_send);
        a.send_meta = st->meta_local(r.slot_send);
        a.send_sb_base = st->meta_sb(r.slot_send);
    }
    if (r.recv) {
        a.step_lo[0] = (uint32_t)r.step_recv; a.step_hi[0] = (uint32_t)(r.step_recv >> 32);
        a.ring_recv = st->ring(r.slot_recv);
        a.recv_meta = st->meta_local(r.slot_recv);
        a.recv_sb_base = st->meta_sb(r.slot_recv);
    }
    return AM_OK;
}

}  // namespace

extern "C" {

const char *am_last_error(void) { return g_last_error; }
const char *am_version(void) { return "asyncmesh-gfx950 0.2 src:" AM_SOURCE_HASH; }

am_status am_workspace_bytes(const am_config *cfg, uint64_t *out_bytes)
{
    if (am_status s = check_config(cfg)) return s;
    if (!out_bytes) return fail(AM_EINVAL, "out_bytes is NULL");
    *out_bytes = am_host::make_layout(*cfg).total;
    return AM_OK;
}

am_status am_d_layout_info(const am_config *cfg, uint32_t *out_replicas_per_block, uint32_t *out_arrays,
                           uint64_t *out_floats_per_array)
{
    if (am_status s = check_config(cfg)) return s;
    uint32_t rb, arrays;
    uint64_t floats;
    am_host::d_layout_shape(*cfg, &rb, &arrays, &floats);
    if (out_replicas_per_block) *out_replicas_per_block = rb;
    if (out_arrays) *out_arrays = arrays;
    if (out_floats_per_array) *out_floats_per_array = floats;
    return AM_OK;
}

}  // extern "C"

namespace {

constexpr uint64_t kSnapshotMagic = 0x414D534E41503033ull;     // "AMSNAP03"

// digest (FNV-1a) of the config fields that shape the ring, the subsets and the caller's arrays
uint64_t config_digest(const am_config &c)
{
    uint64_t fraction_bits;
    std::memcpy(&fraction_bits, &c.fraction, sizeof fraction_bits);
    const uint64_t words[] = { c.n, c.replicas, c.delay, c.avg_interval, c.optimizer, fraction_bits, c.seed,
                               c.subset_granule == 32 ? 32u : 1u, c.subset_kind, c.d_layout, c.ring_cap_lines };
    uint64_t h = 0xCBF29CE484222325ull;
    for (uint64_t w : words)
        for (int b = 0; b < 8; ++b) { h ^= (w >> (8 * b)) & 0xFFu; h *= 0x100000001B3ull; }
    return h;
}

// validates config and buffers and builds the host-side state; clears nothing on the device
am_status create_state(const am_config *cfg, const am_buffers *buf, void *hip_stream, am_state **out)
{
    if (am_status s = check_config(cfg)) return s;
    if (!buf || !out) return fail(AM_EINVAL, "buffers / out is NULL");
    const uint32_t R = cfg->replicas;
    const bool need_m = !(cfg->optimizer == AM_OPT_SGD && cfg->beta1 == 0.f);
    const bool need_v = cfg->optimizer != AM_OPT_SGD;
    const bool need_d = cfg->correction != AM_CORR_NONE;
    const bool need_fwd = cfg->lookahead != 0 || cfg->fwd_dtype == AM_BF16;
    if (!buf->w) return fail(AM_EINVAL, "buffers.w is NULL");
    if (need_m && !buf->m) return fail(AM_EINVAL, "buffers.m is NULL but the optimizer keeps a first moment");
    if (need_v && !buf->v) return fail(AM_EINVAL, "buffers.v is NULL but the optimizer keeps a second moment");
    if (need_d && !buf->d) return fail(AM_EINVAL, "buffers.d is NULL but correction = EMA");
    if (need_fwd && !buf->fwd) return fail(AM_EINVAL, "buffers.fwd is NULL but look-ahead / bf16 forward weights are on");
    const uintptr_t fwd_align = cfg->fwd_dtype == AM_BF16 ? 8 : 16;
    for (uint32_t i = 0; i < R; ++i) {
        if (!buf->w[i]) return fail(AM_EINVAL, "w[%u] is NULL", i);
        if (!aligned(buf->w[i], 16)) return fail(AM_EALIGN, "w[%u] is not 16-byte aligned", i);
        if (need_m) { if (!buf->m[i]) return fail(AM_EINVAL, "m[%u] is NULL", i); if (!aligned(buf->m[i], 16)) return fail(AM_EALIGN, "m[%u] is not 16-byte aligned", i); }
        if (need_v) { if (!buf->v[i]) return fail(AM_EINVAL, "v[%u] is NULL", i); if (!aligned(buf->v[i], 16)) return fail(AM_EALIGN, "v[%u] is not 16-byte aligned", i); }
        if (buf->fwd) { if (!buf->fwd[i]) return fail(AM_EINVAL, "fwd[%u] is NULL", i); if (!aligned(buf->fwd[i], fwd_align)) return fail(AM_EALIGN, "fwd[%u] is not %u-byte aligned", i, (unsigned)fwd_align); }
    }
    uint32_t d_rb = 1, d_arrays = 0;
    uint64_t d_floats = 0;
    if (need_d) {
        am_host::d_layout_shape(*cfg, &d_rb, &d_arrays, &d_floats);
        for (uint32_t k = 0; k < d_arrays; ++k) {
            if (!buf->d[k]) return fail(AM_EINVAL, "d[%u] is NULL", k);
            if (!aligned(buf->d[k], 16)) return fail(AM_EALIGN, "d[%u] is not 16-byte aligned", k);
        }
    }
    const Layout lay = am_host::make_layout(*cfg);
    if (!buf->workspace) return fail(AM_EINVAL, "workspace is NULL");
    if (!aligned(buf->workspace, 256)) return fail(AM_EALIGN, "workspace is not 256-byte aligned");
    if (buf->workspace_bytes < lay.total)
        return fail(AM_ENOMEM, "workspace has %llu bytes, %llu needed", (unsigned long long)buf->workspace_bytes, (unsigned long long)lay.total);

    am_state *st = new (std::nothrow) am_state();
    if (!st) return fail(AM_ENOMEM, "host allocation failed");
    st->cfg = *cfg;
    st->lay = lay;
    st->stream = static_cast<hipStream_t>(hip_stream);
    st->has_fwd = buf->fwd != nullptr;
    st->ws = static_cast<char *>(buf->workspace);
    st->last_t = 0;
    st->next_lines_step = 0;
    st->delay_now = cfg->delay;
    st->overflow_seen = false;
    for (uint32_t i = 0; i < AM_MAX_REPLICAS; ++i) { st->opt_steps[i] = 0; st->mu_product[i] = 1.0; }
    st->threshold = am_host::subset_threshold(cfg->fraction);
    st->profiling = false;
    st->ev_created = st->ev_used = 0;
    st->d_arrays = d_arrays; st->d_rb = d_rb; st->d_floats = d_floats;
    for (uint32_t i = 0; i < AM_MAX_REPLICAS; ++i) {
        st->w[i] = i < R ? buf->w[i] : nullptr;
        st->m[i] = (i < R && need_m) ? buf->m[i] : nullptr;
        st->v[i] = (i < R && need_v) ? buf->v[i] : nullptr;
        st->d[i] = i < d_arrays ? buf->d[i] : nullptr;
        st->fwd[i] = (i < R && buf->fwd) ? buf->fwd[i] : nullptr;
    }

    hipError_t e = hipGetDevice(&st->device);
    int cus = 256;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, st->device);
    if (e != hipSuccess) { delete st; return fail(AM_EHIP, "device query: %s", hipGetErrorString(e)); }
    if (am_status s = resolve_static_scratch(st->device, &st->static_scratch)) { delete st; return s; }
    // the stand-alone kernels stride over the tiles with a fixed number of workgroups per compute unit
    const uint32_t tile_groups = (lay.ntiles + 3) / 4;
    const uint32_t want = (uint32_t)cus * 8u;
    st->grid_sparse = tile_groups < want ? tile_groups : want;
    *out = st;
    return AM_OK;
}

}  // namespace

extern "C" {

am_status am_init_state(const am_config *cfg, const am_buffers *buf, void *hip_stream, am_state **out)
{
    am_state *st = nullptr;
    if (am_status s = create_state(cfg, buf, hip_stream, &st)) return s;
    const uint32_t R = cfg->replicas;
    const bool need_m = st->m[0] != nullptr, need_v = st->v[0] != nullptr;
    const Layout &lay = st->lay;
    hipError_t e = hipSuccess;

    // d^0 = 0 and zero moments; clear flags, offsets and ring
    const size_t bytes = (size_t)cfg->n * sizeof(float);
    for (uint32_t i = 0; i < R && e == hipSuccess; ++i) {
        if (need_m) e = hipMemsetAsync(st->m[i], 0, bytes, st->stream);
        if (need_v && e == hipSuccess) e = hipMemsetAsync(st->v[i], 0, bytes, st->stream);
    }
    for (uint32_t k = 0; k < st->d_arrays && e == hipSuccess; ++k)
        e = hipMemsetAsync(st->d[k], 0, (size_t)st->d_floats * sizeof(float), st->stream);
    if (e == hipSuccess) e = hipMemsetAsync(st->ws, 0, lay.total, st->stream);
    if (e != hipSuccess) { delete st; return fail(AM_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); }
    *out = st;
    return AM_OK;
}

am_status am_export_state(const am_state *st, am_snapshot *out)
{
    if (!st || !out) return fail(AM_EINVAL, "NULL argument");
    out->magic = kSnapshotMagic;
    out->config_digest = config_digest(st->cfg);
    out->last_t = st->last_t;
    out->next_lines_step = st->next_lines_step;
    for (uint32_t i = 0; i < AM_MAX_REPLICAS; ++i) { out->opt_steps[i] = st->opt_steps[i]; out->mu_product[i] = st->mu_product[i]; }
    out->delay_now = st->delay_now;
    out->reserved = 0;
    return AM_OK;
}

am_status am_resume_state(const am_config *cfg, const am_buffers *buf, void *hip_stream,
                          const am_snapshot *snapshot, am_state **out)
{
    if (am_status s = check_config(cfg)) return s;
    if (!snapshot) return fail(AM_EINVAL, "snapshot is NULL");
    if (snapshot->magic != kSnapshotMagic) return fail(AM_EINVAL, "snapshot has an unknown layout (magic %016llx)", (unsigned long long)snapshot->magic);
    if (snapshot->config_digest != config_digest(*cfg)) return fail(AM_EINVAL, "snapshot was exported under a different config (n, replicas, delay, avg_interval, optimizer, fraction, seed, subset rule, d_layout or ring_cap_lines differ)");
    if (snapshot->delay_now > cfg->delay) return fail(AM_EINVAL, "snapshot delay %u exceeds the configured delay %u", snapshot->delay_now, cfg->delay);
    for (uint32_t i = 0; i < AM_MAX_REPLICAS; ++i)
        if (!(snapshot->mu_product[i] >= 0.0 && snapshot->mu_product[i] <= 1.0)) return fail(AM_EINVAL, "snapshot mu_product[%u]=%g not in [0, 1]", i, snapshot->mu_product[i]);
    am_state *st = nullptr;
    if (am_status s = create_state(cfg, buf, hip_stream, &st)) return s;
    st->last_t = snapshot->last_t;
    st->next_lines_step = snapshot->next_lines_step;
    for (uint32_t i = 0; i < AM_MAX_REPLICAS; ++i) { st->opt_steps[i] = snapshot->opt_steps[i]; st->mu_product[i] = snapshot->mu_product[i]; }
    st->delay_now = snapshot->delay_now;
    *out = st;
    return AM_OK;
}

am_status am_step(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t, float grad_scale)
{
    return am_step_scaled(st, t, grads, lr, lambda_t, grad_scale, nullptr);
}

am_status am_grad_sqnorm(am_state *st, const void *const *grads, double *dev_out)
{
    if (!st || !grads || !dev_out) return fail(AM_EINVAL, "NULL argument");
    if (!aligned(dev_out, 8)) return fail(AM_EALIGN, "dev_out is not 8-byte aligned");
    const am_config &c = st->cfg;
    const uintptr_t galign = c.grad_dtype == AM_BF16 ? 8 : 16;
    am::NormArgs a;
    std::memset(&a, 0, sizeof a);
    for (uint32_t i = 0; i < c.replicas; ++i) {
        if (!grads[i]) return fail(AM_EINVAL, "grads[%u] is NULL", i);
        if (!aligned(grads[i], galign)) return fail(AM_EALIGN, "grads[%u] is not %u-byte aligned", i, (unsigned)galign);
        a.g[i] = grads[i];
    }
    a.n = c.n; a.replicas = c.replicas; a.is_bf16 = c.grad_dtype == AM_BF16;
    const uint64_t want = ((c.n + 3) / 4 + 255) / 256;
    const uint32_t blocks = (uint32_t)(want < 1024 ? want : 1024);
    am::k_sqnorm_partial<<<dim3(blocks, c.replicas), 256, 0, st->stream>>>(a, st->reduce_partials());
    AM_HIP(hipGetLastError());
    am::k_sqnorm_final<<<c.replicas, 256, 0, st->stream>>>(st->reduce_partials(), blocks, dev_out);
    AM_HIP(hipGetLastError());
    return AM_OK;
}

}  // extern "C"

namespace {

// One step (active == nullptr: every replica steps and its optimizer step count becomes t) or one
// tick of the heterogeneous set-up (bit i of *active: replica i makes a local step and counts it).
am_status step_impl(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t,
                    float grad_scale, const float *dev_replica_scale, const uint32_t *active)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (st->overflow_seen) return fail(AM_EOVERFLOW, "a subset did not fit its ring slot (reported by am_read_flags): the state no longer follows the method");
    if (!aligned(dev_replica_scale, 4)) return fail(AM_EALIGN, "dev_replica_scale is not 4-byte aligned");
    if (!grads) return fail(AM_EINVAL, "grads is NULL");
    if (t != st->last_t + 1) return fail(AM_EORDER, "step %llu after step %llu", (unsigned long long)t, (unsigned long long)st->last_t);
    if (!(lambda_t >= 0.f && lambda_t <= 1.f)) return fail(AM_EINVAL, "lambda_t=%g not in [0, 1]", lambda_t);
    if (!std::isfinite(lr) || !std::isfinite(grad_scale)) return fail(AM_EINVAL, "lr / grad_scale not finite");
    const am_config &c = st->cfg;
    const uint32_t all = c.replicas == 32 ? 0xFFFFFFFFu : ((1u << c.replicas) - 1u);
    if (active && (*active & ~all)) return fail(AM_EINVAL, "active_mask=%08x names replicas beyond %u", *active, c.replicas);
    const uint32_t mask = active ? *active : all;
    const uintptr_t galign = c.grad_dtype == AM_BF16 ? 8 : 16;
    for (uint32_t i = 0; i < c.replicas; ++i) {
        if (!((mask >> i) & 1u)) continue;                       // an idle replica's gradient is not read
        if (!grads[i]) return fail(AM_EINVAL, "grads[%u] is NULL", i);
        if (!aligned(grads[i], galign)) return fail(AM_EALIGN, "grads[%u] is not %u-byte aligned", i, (unsigned)galign);
    }

    // the two events that bracket the kernel exist before anything is enqueued
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    const bool timed = st->profiling && st->ev_used + 2 <= 2 * kMaxProfiledLaunches;
    if (timed) {
        while (st->ev_created < st->ev_used + 2) {
            AM_HIP(hipEventCreate(&st->ev_pool[st->ev_created]));
            ++st->ev_created;
        }
        ev0 = st->ev_pool[st->ev_used];
        ev1 = st->ev_pool[st->ev_used + 1];
    }

    am::StepArgs a;
    std::memset(&a, 0, sizeof a);
    const am_host::Blocks &B = st->lay.blocks;
    auto slot = [&B](uint32_t i) { return 8u * (i / B.rb) + i % B.rb; };     // where replica i's record sits
    for (uint32_t i = 0; i < c.replicas; ++i) {
        am::ReplicaArgs &r = a.rep[slot(i)];
        r.w = st->w[i]; r.m = st->m[i]; r.v = st->v[i];
        r.fwd = st->fwd[i];
        r.g = ((mask >> i) & 1u) ? grads[i] : nullptr;                      // NULL = idle in this launch
    }
    a.lookahead = c.lookahead != 0; a.gamma = (double)c.gamma;
    a.replica_scale = dev_replica_scale;
    const double gs = (double)grad_scale;        // folded into the coefficients that multiply g

    // per-step scalars, evaluated once in double; those that depend on a replica's own step count per replica
    const double b1 = c.beta1, b2 = c.beta2, lrd = lr, wd = c.weight_decay;
    uint64_t steps_next[AM_MAX_REPLICAS];
    double mu_prod_next[AM_MAX_REPLICAS];
    a.c_wd = lrd * wd;
    a.eps = (double)c.eps;
    if (c.optimizer == AM_OPT_SGD) {
        a.a_m = b1; a.b_m = gs;
    } else {
        a.a_m = b1; a.b_m = (1.0 - b1) * gs;
        a.a_v = b2; a.b_v = (1.0 - b2) * gs * gs;
    }
    for (uint32_t i = 0; i < c.replicas; ++i) {
        steps_next[i] = st->opt_steps[i];
        mu_prod_next[i] = st->mu_product[i];
        if (!((mask >> i) & 1u)) continue;
        const uint64_t k = active ? st->opt_steps[i] + 1 : t;
        steps_next[i] = k;
        if (c.optimizer == AM_OPT_SGD) {
            a.rep[slot(i)].c_m = lrd; a.rep[slot(i)].c_g = lrd * gs;
            continue;
        }
        const double bc1 = 1.0 - std::pow(b1, (double)k), bc2 = 1.0 - std::pow(b2, (double)k);
        a.rep[slot(i)].c_v = 1.0 / std::sqrt(bc2);
        if (c.optimizer == AM_OPT_ADAMW) {
            a.rep[slot(i)].c_g = 0.0; a.rep[slot(i)].c_m = lrd / bc1;
        } else {
            const double mu_t = b1 * (1.0 - 0.5 * std::pow(0.96, (double)k * c.momentum_decay));
            const double mu_t1 = b1 * (1.0 - 0.5 * std::pow(0.96, (double)(k + 1) * c.momentum_decay));
            mu_prod_next[i] = st->mu_product[i] * mu_t;
            a.rep[slot(i)].c_g = lrd * (1.0 - mu_t) / (1.0 - mu_prod_next[i]) * gs;
            a.rep[slot(i)].c_m = lrd * mu_t1 / (1.0 - mu_prod_next[i] * mu_t1);
        }
    }

    for (uint32_t b = 0; b < B.nblocks; ++b)                  // slots of absent replicas: loads through them must be harmless
        for (uint32_t k = 0; k < B.rb; ++k)
            if (b * B.rb + k >= c.replicas) a.rep[8u * b + k] = a.rep[8u * b];

    const Round r = plan_round(st, t);
    if (am_status s = fill_averaging(st, t, lambda_t, r, a)) return s;

    const bool do_next = (t + 1) % c.avg_interval == 0;      // the next step sends: size its tiles on the way
    a.do_next = do_next;
    if (do_next) {
        a.step_lo[2] = (uint32_t)(t + 1); a.step_hi[2] = (uint32_t)((t + 1) >> 32);
        a.next_lines = st->next_lines();
    }

    if (timed) AM_HIP(hipEventRecord(ev0, st->stream));
    am_status s;
    if (c.optimizer == AM_OPT_SGD) s = c.beta1 == 0.f ? launch_step_grad<am::kOptSgdPlain>(st, a) : launch_step_grad<am::kOptSgdMomentum>(st, a);
    else s = launch_step_grad<am::kOptAdam>(st, a);
    if (s) return s;
    if (timed) {
        AM_HIP(hipEventRecord(ev1, st->stream));
        st->ev_used += 2;
    }
    st->last_t = t;
    if (do_next) st->next_lines_step = t + 1;
    for (uint32_t i = 0; i < c.replicas; ++i) { st->opt_steps[i] = steps_next[i]; st->mu_product[i] = mu_prod_next[i]; }
    return AM_OK;
}

}  // namespace

extern "C" {

am_status am_step_scaled(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t,
                         float grad_scale, const float *dev_replica_scale)
{
    return step_impl(st, t, grads, lr, lambda_t, grad_scale, dev_replica_scale, nullptr);
}

am_status am_step_masked(am_state *st, uint64_t t, const void *const *grads, float lr, float lambda_t,
                         float grad_scale, const float *dev_replica_scale, uint32_t active_mask)
{
    return step_impl(st, t, grads, lr, lambda_t, grad_scale, dev_replica_scale, &active_mask);
}

am_status am_sparse_average(am_state *st, uint64_t t, float lambda_t)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (st->overflow_seen) return fail(AM_EOVERFLOW, "a subset did not fit its ring slot (reported by am_read_flags): the state no longer follows the method");
    if (t != st->last_t + 1) return fail(AM_EORDER, "step %llu after step %llu", (unsigned long long)t, (unsigned long long)st->last_t);
    if (!(lambda_t >= 0.f && lambda_t <= 1.f)) return fail(AM_EINVAL, "lambda_t=%g not in [0, 1]", lambda_t);
    const Round r = plan_round(st, t);
    const bool do_next = (t + 1) % st->cfg.avg_interval == 0;      // the next step sends: size its tiles on the way
    if (r.send) {
        am::StepArgs a;
        std::memset(&a, 0, sizeof a);
        for (uint32_t i = 0; i < st->cfg.replicas; ++i) a.rep[8u * (i / st->lay.blocks.rb) + i % st->lay.blocks.rb].w = st->w[i];
        if (am_status s = fill_averaging(st, t, lambda_t, r, a)) return s;
        a.do_next = do_next;
        if (do_next) {
            a.step_lo[2] = (uint32_t)(t + 1); a.step_hi[2] = (uint32_t)((t + 1) >> 32);
            a.next_lines = st->next_lines();
        }
        const bool dil = st->cfg.d_layout == AM_D_INTERLEAVED && a.ema;
        const bool tau0 = r.recv && r.same_slot;           // the average is of this call's own values
        if (am_status s = dil ? (tau0 ? launch_average<true, true>(st, a) : launch_average<true, false>(st, a))
                              : (tau0 ? launch_average<false, true>(st, a) : launch_average<false, false>(st, a))) return s;
        if (do_next) st->next_lines_step = t + 1;
    }
    st->last_t = t;
    return AM_OK;
}

am_status am_lookahead(void *out, uint32_t out_dtype, const float *w, const float *w_prev, uint64_t n, float gamma, void *hip_stream)
{
    if (!out || !w || !w_prev) return fail(AM_EINVAL, "NULL pointer");
    if (out_dtype > AM_BF16) return fail(AM_EINVAL, "unknown dtype");
    if (!std::isfinite(gamma)) return fail(AM_EINVAL, "gamma not finite");
    if (!aligned(w, 16) || !aligned(w_prev, 16) || !aligned(out, out_dtype == AM_BF16 ? 8 : 16)) return fail(AM_EALIGN, "pointer not aligned");
    if (n == 0) return AM_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint64_t ngroups = (n + 3) / 4;
    const uint64_t blocks_needed = (ngroups + 255) / 256;
    // one group per thread (measured on MI355X: a one-shot grid streams faster than a few resident workgroups
    // that loop); the kernel's loop takes over only beyond 2^31 - 1 workgroups, which no accepted n reaches
    const uint32_t grid = (uint32_t)(blocks_needed < 0x7FFFFFFFull ? blocks_needed : 0x7FFFFFFFull);
    if (out_dtype == AM_BF16) am::k_lookahead<true><<<grid, 256, 0, s>>>(out, w, w_prev, n, (double)gamma);
    else am::k_lookahead<false><<<grid, 256, 0, s>>>(out, w, w_prev, n, (double)gamma);
    AM_HIP(hipGetLastError());
    return AM_OK;
}

am_status am_subset_indices(am_state *st, uint64_t t, uint64_t *dev_out, uint64_t capacity, uint64_t *dev_count)
{
    if (am_status s = check_index_list_args(st, dev_out, capacity, dev_count)) return s;
    const uint32_t meta_slot = st->lay.slots;        // the metadata block after the ring slots' own
    return launch_index_list(st, t, st->meta_local(meta_slot), st->meta_sb(meta_slot), dev_out, capacity, dev_count);
}

am_status am_subset_indices_static(am_state *st, uint64_t t, uint64_t *dev_out, uint64_t capacity, uint64_t *dev_count)
{
    if (am_status s = check_index_list_args(st, dev_out, capacity, dev_count)) return s;
    if (st->cfg.n > kStaticMaxN)
        return fail(AM_EINVAL, "n=%llu exceeds the %llu coordinates the static scratch covers; use am_subset_indices",
                    (unsigned long long)st->cfg.n, (unsigned long long)kStaticMaxN);
    int device = -1;
    AM_HIP(hipGetDevice(&device));
    if (device != st->device) return fail(AM_EINVAL, "device %d is current, the state lives on device %d", device, st->device);
    uint32_t *base = st->static_scratch;             // looked up at am_init_state / am_resume_state
    return launch_index_list(st, t, base, base + kStaticMaxTiles, dev_out, capacity, dev_count);
}

am_status am_set_delay(am_state *st, uint32_t tau)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (tau > st->cfg.delay) return fail(AM_EINVAL, "delay %u exceeds the ring depth the state was created with (%u)", tau, st->cfg.delay);
    st->delay_now = tau;
    return AM_OK;
}

am_status am_diagnostics(am_state *st, double *dev_out3)
{
    if (!st || !dev_out3) return fail(AM_EINVAL, "NULL argument");
    if (!aligned(dev_out3, 8)) return fail(AM_EALIGN, "dev_out3 is not 8-byte aligned");
    am::DiagArgs a;
    std::memset(&a, 0, sizeof a);
    a.has_d = st->d_arrays != 0;
    a.d_stride = st->d_rb;
    for (uint32_t i = 0; i < st->cfg.replicas; ++i) a.w[i] = st->w[i];
    for (uint32_t k = 0; k < st->d_arrays; ++k) a.d[k] = st->d[k];          // per replica, or (interleaved) per block
    a.n = st->cfg.n; a.replicas = st->cfg.replicas;
    const uint64_t want = ((st->cfg.n + 3) / 4 + 255) / 256;               // a thread takes groups of 4 coordinates
    const uint32_t blocks = (uint32_t)(want < 4096 ? want : 4096);          // 3 doubles each in the partials area (32 x 1024 doubles)
    if (a.replicas <= 8) am::k_diag_partial<8><<<blocks, 256, 0, st->stream>>>(a, st->reduce_partials());
    else if (a.replicas <= 16) am::k_diag_partial<16><<<blocks, 256, 0, st->stream>>>(a, st->reduce_partials());
    else am::k_diag_partial<32><<<blocks, 256, 0, st->stream>>>(a, st->reduce_partials());
    AM_HIP(hipGetLastError());
    am::k_diag_final<<<1, 256, 0, st->stream>>>(st->reduce_partials(), blocks, st->cfg.n, dev_out3);
    AM_HIP(hipGetLastError());
    return AM_OK;
}

am_status am_read_flags(am_state *st, uint32_t *out_flags)
{
    if (!st || !out_flags) return fail(AM_EINVAL, "NULL argument");
    AM_HIP(hipMemcpyAsync(out_flags, st->flags(), sizeof(uint32_t), hipMemcpyDeviceToHost, st->stream));
    AM_HIP(hipStreamSynchronize(st->stream));
    if (*out_flags & 1u) st->overflow_seen = true;
    return AM_OK;
}

am_status am_set_profiling(am_state *st, int on)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (on && !st->profiling) st->ev_used = 0;
    st->profiling = on != 0;
    return AM_OK;
}

am_status am_get_profile_times(am_state *st, float *out_ms, uint64_t capacity, uint64_t *out_launches)
{
    if (!st || !out_launches || (!out_ms && capacity)) return fail(AM_EINVAL, "NULL argument");
    AM_HIP(hipStreamSynchronize(st->stream));
    for (uint32_t k = 0; k + 1 < st->ev_used; k += 2) {
        float ms = 0.f;
        AM_HIP(hipEventElapsedTime(&ms, st->ev_pool[k], st->ev_pool[k + 1]));
        if (k / 2 < capacity) out_ms[k / 2] = ms;
    }
    *out_launches = st->ev_used / 2;
    st->ev_used = 0;
    return AM_OK;
}

am_status am_get_profile(am_state *st, double *out_kernel_ms, uint64_t *out_launches)
{
    if (!st || !out_kernel_ms || !out_launches) return fail(AM_EINVAL, "NULL argument");
    AM_HIP(hipStreamSynchronize(st->stream));
    double total = 0.0;
    for (uint32_t k = 0; k + 1 < st->ev_used; k += 2) {
        float ms = 0.f;
        AM_HIP(hipEventElapsedTime(&ms, st->ev_pool[k], st->ev_pool[k + 1]));
        total += ms;
    }
    *out_kernel_ms = total;
    *out_launches = st->ev_used / 2;
    st->ev_used = 0;
    return AM_OK;
}

am_status am_ring_info(const am_state *st, uint64_t *out_capacity, uint32_t *out_slots)
{
    if (!st) return fail(AM_EINVAL, "state is NULL");
    if (out_capacity) *out_capacity = st->lay.cap_lines * am::kLineFloats;
    if (out_slots) *out_slots = st->lay.slots;
    return AM_OK;
}

am_status am_destroy(am_state *st)
{
    if (!st) return AM_OK;
    for (uint32_t k = 0; k < st->ev_created; ++k) (void)hipEventDestroy(st->ev_pool[k]);
    delete st;
    return AM_OK;
}

}  // extern "C"
