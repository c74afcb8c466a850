// Live intervals, linear-scan buffer assignment and workspace layout of a flat instruction
// list (Sec. "Phase 4: IR Analysis & Optimization").  Host code only: nothing here touches
// the GPU.
#include "plan.hpp"

#include <algorithm>
#include <functional>
#include <queue>
#include <utility>
#include <vector>

#include "../../include/forge.h"

namespace forge {

void plan_liveness(int n_instr, const int* out_reg, const int* in_begin, const int* in_regs,
                   int n_regs, int* start, int* end) {
  std::fill(start, start + n_regs, -1);
  std::fill(end, end + n_regs, -1);
  auto touch = [&](int r, int j) {
    if (start[r] < 0) start[r] = j;
    end[r] = j;
  };
  for (int j = 0; j < n_instr; ++j) {
    for (int i = in_begin[j]; i < in_begin[j + 1]; ++i) touch(in_regs[i], j);
    if (out_reg[j] >= 0) touch(out_reg[j], j);
  }
}

// Alg. "Linear-Scan Buffer Allocation" as an event sweep: the intervals arrive by ascending start;
// the ones still holding a buffer wait in a heap keyed by their end, so the arrivals' expiry step
// pops exactly those that ended strictly before the new start; released buffers wait in a second
// heap keyed by their number.  The algorithm only says that a free buffer is popped: which one is
// this library's choice (the lowest-numbered), documented at the entry point.
int plan_linear_scan(int n_regs, const int* start, const int* end, int* reg_to_buf) {
  std::vector<int> order;
  order.reserve(n_regs);
  for (int r = 0; r < n_regs; ++r) {
    reg_to_buf[r] = -1;
    if (start[r] >= 0) order.push_back(r);
  }
  std::sort(order.begin(), order.end(),
            [&](int a, int b) { return start[a] != start[b] ? start[a] < start[b] : a < b; });
  typedef std::pair<int, int> Held;   // (end of the interval, its buffer)
  std::priority_queue<Held, std::vector<Held>, std::greater<Held>> holding;
  std::priority_queue<int, std::vector<int>, std::greater<int>> idle;
  int n_bufs = 0;
  for (int r : order) {
    while (!holding.empty() && holding.top().first < start[r]) {
      idle.push(holding.top().second);
      holding.pop();
    }
    int b;
    if (!idle.empty()) {
      b = idle.top();
      idle.pop();
    } else {
      b = n_bufs++;
    }
    reg_to_buf[r] = b;
    holding.push(Held(end[r], b));
  }
  return n_bufs;
}

size_t plan_workspace(int n_regs, const int* start, const int* end, const size_t* nbytes,
                      size_t* offset, int* n_bufs) {
  std::vector<char> placed(n_regs, 0);
  std::vector<int> members, s, e, buf;
  size_t base = 0;
  int total_bufs = 0;
  std::fill(offset, offset + n_regs, (size_t)-1);
  auto single = [&](int r) { return start[r] == end[r]; };
  for (int r0 = 0; r0 < n_regs; ++r0) {
    if (start[r0] < 0 || placed[r0]) continue;
    // the group of r0: every single-instruction register, or every longer-lived one of its size
    members.clear();
    size_t size = 0;
    for (int r = r0; r < n_regs; ++r) {
      if (start[r] < 0 || placed[r]) continue;
      if (single(r0) ? single(r) : (!single(r) && nbytes[r] == nbytes[r0])) {
        members.push_back(r);
        size = std::max(size, nbytes[r]);
      }
    }
    const int n = (int)members.size();
    s.resize(n); e.resize(n); buf.resize(n);
    for (int i = 0; i < n; ++i) { s[i] = start[members[i]]; e[i] = end[members[i]]; }
    const int m = plan_linear_scan(n, s.data(), e.data(), buf.data());
    const size_t stride = (size + 255) / 256 * 256;
    for (int i = 0; i < n; ++i) {
      offset[members[i]] = base + (size_t)buf[i] * stride;
      placed[members[i]] = 1;
    }
    base += (size_t)m * stride;
    total_bufs += m;
  }
  if (n_bufs != nullptr) *n_bufs = total_bufs;
  return base;
}

}  // namespace forge

namespace {

bool program_ok(int n_instr, const int* out_reg, const int* in_begin, const int* in_regs, int n_regs) {
  if (n_instr < 0 || n_regs < 0 || out_reg == nullptr || in_begin == nullptr) return false;
  if (in_begin[0] != 0) return false;
  for (int j = 0; j < n_instr; ++j) {
    if (in_begin[j + 1] < in_begin[j]) return false;
    if (out_reg[j] < -1 || out_reg[j] >= n_regs) return false;
  }
  if (in_begin[n_instr] > 0 && in_regs == nullptr) return false;
  for (int i = 0; i < in_begin[n_instr]; ++i)
    if (in_regs[i] < 0 || in_regs[i] >= n_regs) return false;
  return true;
}

bool intervals_ok(int n_regs, const int* start, const int* end) {
  if (n_regs < 0 || start == nullptr || end == nullptr) return false;
  for (int r = 0; r < n_regs; ++r) {
    if (start[r] < 0 ? end[r] >= 0 : end[r] < start[r]) return false;
  }
  return true;
}

}  // namespace

extern "C" {

forge_status forge_plan_liveness(int n_instr, const int* out_reg, const int* in_begin,
                                 const int* in_regs, int n_regs, int* start, int* end) {
  if (start == nullptr || end == nullptr || !program_ok(n_instr, out_reg, in_begin, in_regs, n_regs))
    return FORGE_ERR_INVALID_ARG;
  forge::plan_liveness(n_instr, out_reg, in_begin, in_regs, n_regs, start, end);
  return FORGE_OK;
}

forge_status forge_plan_dead_after(int n_regs, const int* end, int n_instr, int* dead_begin,
                                   int* dead_regs) {
  if (n_regs < 0 || n_instr < 0 || end == nullptr || dead_begin == nullptr || dead_regs == nullptr)
    return FORGE_ERR_INVALID_ARG;
  for (int r = 0; r < n_regs; ++r)
    if (end[r] >= n_instr) return FORGE_ERR_INVALID_ARG;
  std::fill(dead_begin, dead_begin + n_instr + 1, 0);
  for (int r = 0; r < n_regs; ++r)
    if (end[r] >= 0) ++dead_begin[end[r] + 1];
  for (int j = 0; j < n_instr; ++j) dead_begin[j + 1] += dead_begin[j];
  std::vector<int> fill(dead_begin, dead_begin + n_instr);
  for (int r = 0; r < n_regs; ++r)
    if (end[r] >= 0) dead_regs[fill[end[r]]++] = r;
  return FORGE_OK;
}

forge_status forge_plan_linear_scan(int n_regs, const int* start, const int* end, int* reg_to_buf,
                                    int* n_bufs) {
  if (reg_to_buf == nullptr || n_bufs == nullptr || !intervals_ok(n_regs, start, end))
    return FORGE_ERR_INVALID_ARG;
  *n_bufs = forge::plan_linear_scan(n_regs, start, end, reg_to_buf);
  return FORGE_OK;
}

forge_status forge_plan_workspace(int n_regs, const int* start, const int* end,
                                  const size_t* nbytes, size_t* offset, size_t* total_bytes,
                                  int* n_bufs) {
  if (nbytes == nullptr || offset == nullptr || total_bytes == nullptr || !intervals_ok(n_regs, start, end))
    return FORGE_ERR_INVALID_ARG;
  *total_bytes = forge::plan_workspace(n_regs, start, end, nbytes, offset, n_bufs);
  return FORGE_OK;
}

}  // extern "C"
