// C entry points over the library's host-side arithmetic (am_host_logic.h: no HIP inside), so that a
// test on a machine without a GPU can drive it directly.  Built by tests/test_host_logic.py with g++.
#include "../paper_2601_22442_amd/csrc/am_host_logic.h"

extern "C" {

uint64_t hl_threshold(double p) { return am_host::subset_threshold(p); }
uint64_t hl_stratified_block(double p) { return am_host::stratified_block(p); }

void hl_blocks(uint32_t replicas, uint32_t *rb, uint32_t *rb_shift, uint32_t *nblocks)
{
    const am_host::Blocks b = am_host::block_geometry(replicas);
    *rb = b.rb; *rb_shift = b.rb_shift; *nblocks = b.nblocks;
}

uint64_t hl_capacity(uint64_t ntiles, double p, uint32_t rb, int by_line, uint64_t strat_block)
{
    return am_host::slot_capacity_lines(ntiles, p, rb, by_line != 0, strat_block);
}

// out[0..11]: ntiles, nsb, slots, cap_lines, off_flags, off_reduce, off_next, off_meta, meta_stride, off_ring, ring_stride, total
// out[12]: meta_sb_off
void hl_layout(const am_config *c, uint64_t *out)
{
    const am_host::Layout L = am_host::make_layout(*c);
    const uint64_t v[] = { L.ntiles, L.nsb, L.slots, L.cap_lines, L.off_flags, L.off_reduce, L.off_next, L.off_meta,
                           L.meta_stride, L.off_ring, L.ring_stride, L.total, L.meta_sb_off };
    for (unsigned k = 0; k < sizeof v / sizeof v[0]; ++k) out[k] = v[k];
}

// out: send, recv, same_slot, slot_send, slot_recv, step_recv
void hl_plan_round(uint64_t K, uint64_t depth, uint64_t tau, uint64_t t, uint64_t *out)
{
    const am_host::Round r = am_host::plan_round(K, depth, tau, t);
    out[0] = r.send; out[1] = r.recv; out[2] = r.same_slot; out[3] = r.slot_send; out[4] = r.slot_recv; out[5] = r.step_recv;
}

void hl_d_shape(const am_config *c, uint32_t *rb, uint32_t *arrays, uint64_t *floats) { am_host::d_layout_shape(*c, rb, arrays, floats); }

}  // extern "C"
