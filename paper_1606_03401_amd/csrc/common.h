// Internal declarations shared by the planner and the executor.  Not part of the ABI.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "mebptt.h"

namespace mebptt {

// Thread-local text of the last error; set_error returns `code` so call sites can `return` it.
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Row-major [(t+1) x (m+1)] tables as exposed through the ABI.
struct Tables {
  int32_t t = 0, m = 0;
  std::vector<int64_t> C, C1, C2;   // C1/C2: MSM only
  std::vector<int32_t> D, D1, D2;   // D: HSM/ISM; D1/D2: MSM only
  std::vector<uint8_t> Hc;          // MSM only
  size_t idx(int32_t tt, int32_t mm) const { return (size_t)tt * (size_t)(m + 1) + (size_t)mm; }
};

}  // namespace mebptt

struct mebptt_plan_s {
  int32_t t = 0, m = 0, kind = 0, alpha = 0, beta = 0;
  mebptt::Tables tab;
  std::vector<mebptt_op> ops;
  int64_t forward_ops = 0;
  int64_t backward_ops = 0;
  int32_t peak = 0;   // in budget units of `kind`
  bool from_policy = false;   // flattened from a caller-supplied decision list: no tables
};
