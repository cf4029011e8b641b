// Unit descriptors of a launch group that is too large for the kernel arguments (more than kInlineUnits units).
//
// The library neither allocates nor copies from host memory (a call must stay capturable into a HIP graph and must
// not wait for the device), so the descriptors reach the workspace the way everything else reaches the device: as
// kernel arguments.  One tiny launch carries kInlineUnits descriptors by value and its threads store them; the
// group's kernels, later on the same stream, read them from there (UnitTable::unit).
#include "kvs_device.h"

namespace kvs {
namespace {

struct UnitBatch {
  Unit u[kInlineUnits];
};

__global__ __launch_bounds__(kInlineUnits) void unit_table_kernel(const UnitBatch batch, int n, Unit* __restrict__ dst) {
  const int i = threadIdx.x;
  if (i < n) dst[i] = batch.u[i];
}

}  // namespace

hipError_t launch_unit_table(const Unit* units, int n_units, Unit* dst, hipStream_t stream) {
  for (int first = 0; first < n_units; first += kInlineUnits) {
    const int n = n_units - first < kInlineUnits ? n_units - first : kInlineUnits;
    UnitBatch batch;
    for (int i = 0; i < kInlineUnits; ++i) batch.u[i] = units[first + (i < n ? i : 0)];
    hipLaunchKernelGGL(unit_table_kernel, dim3(1), dim3(kInlineUnits), 0, stream, batch, n, dst + first);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace kvs
