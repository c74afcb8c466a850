// Static buffer plan of a flat instruction list (Sec. "Phase 4: IR Analysis & Optimization"):
// live intervals (Eq. "liveness"), linear-scan assignment of virtual registers to buffers
// (Alg. "Linear-Scan Buffer Allocation"), and the byte layout of one workspace built on it.
// Host code only.
#pragma once
#include <cstddef>
#include <vector>

namespace forge {

// Instruction j writes out_reg[j] (or -1) and reads in_regs[in_begin[j] .. in_begin[j+1]).
// start[r] = index of the first instruction that mentions register r (its writer, in a
// well-formed program), end[r] = index of the last one; both -1 for a register never mentioned.
void plan_liveness(int n_instr, const int* out_reg, const int* in_begin, const int* in_regs,
                   int n_regs, int* start, int* end);

// Intervals are visited by ascending start (ties: ascending register number).  Before each one,
// intervals whose end lies strictly before its start give their buffer back; the interval takes
// the lowest-numbered free buffer, else a new one (numbered 0, 1, ... in creation order).
// Registers with start < 0 get buffer -1.  Returns the number of buffers.
int plan_linear_scan(int n_regs, const int* start, const int* end, int* reg_to_buf);

// Byte layout: registers of equal byte size form a group, except that all registers living within
// one instruction (start == end: scratch areas) form a single group sized to its largest member;
// each group is assigned by its own linear scan, groups follow each other in the order of their
// first register; every buffer of a group spans the group's size rounded up to 256 bytes.  offset[r] = (size_t)-1 for registers
// with start < 0.  Returns the total size; *n_bufs = buffers over all groups.
size_t plan_workspace(int n_regs, const int* start, const int* end, const size_t* nbytes,
                      size_t* offset, int* n_bufs);

}  // namespace forge
