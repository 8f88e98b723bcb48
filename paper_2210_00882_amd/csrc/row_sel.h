// Row selection shared by the learner's kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace msrl {

// The rows a learner call works on, inside the caller's arrays: logical row r is array row
//   row0 + r                                              (count == 0: consecutive rows)
//   ((row0 + r) / count) * group + first + (row0 + r) % count   (the agents first .. first+count-1 of
//                                                          every group of `group` rows: one role)
struct RowSel {
  int64_t row0;
  int32_t group, first, count;
  __host__ __device__ int64_t at(int64_t r) const {
    const int64_t q = row0 + r;
    return count == 0 ? q : (q / count) * group + first + q % count;
  }
};

}  // namespace msrl
