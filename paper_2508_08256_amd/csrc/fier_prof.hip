// Tuning build only (`python -m paper_2508_08256_amd.build --prof` -> libfier_prof.so, compiled with
// -DFIER_PROF_ENABLE): storage for the kernels' optional time stamps (FIER_PROF / FIER_PROF_WG in fier_dev.h)
// and the host calls that read and clear them.  Not part of libfier.so.
#include <hip/hip_runtime.h>
__device__ unsigned long long fier_prof_slots[64];
__device__ unsigned long long fier_prof_wg[8][4096];
extern "C" int fier_prof_read(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fier_prof_slots), sizeof(unsigned long long) * 64);
}
extern "C" int fier_prof_read_wg(unsigned long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fier_prof_wg), sizeof(unsigned long long) * 8 * 4096);
}
extern "C" int fier_prof_reset() {
  static unsigned long long zero[8 * 4096];
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(fier_prof_wg), zero, sizeof(zero));
}
