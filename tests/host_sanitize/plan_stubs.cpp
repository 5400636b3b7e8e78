// plan_stubs.cpp — stand-ins for the kernel-geometry predicates that the host planner (ae_plan.cpp) asks of the HIP
// translation units, so that the planner can be built and run WITHOUT the GPU toolchain under AddressSanitizer /
// UBSan (tests/test_host_sanitizers.py).  They answer like the real ones for the shapes of the five workloads
// (thin first / last layers, MFMA weight gradients) and return sizes of the right order; the planner's own
// arithmetic (parsing, shape inference, offsets, workspace sums) is what the sanitizer run exercises.
#include "ae_internal.h"

namespace ae {
int plane_sums_split(int64_t hw) { return hw >= 4096 ? 8 : 1; }
int64_t thin_wfrag_bytes(int cw) { return (int64_t)cw * 16 * 2 * 3; }
bool thin_in_supported(int ct, int cw, int k, int up) { return ct >= 1 && ct <= 4 && k == 3 && !up && cw >= 1; }
int64_t thin_out_wz_bytes(int ct, int cw) { return (int64_t)ct * cw * 9 * 2 + 256; }
bool thin_out_supported(int ct, int cw, int k, int dtype) { return ct >= 1 && ct <= 4 && k == 3 && cw >= 1 && (dtype == 0 || dtype == 1); }
int thin_in_mfma_blocks(int n, int h, int w) { return (int)(((int64_t)n * h * w + 255) / 256); }
bool conv_up_dgrad_usable(const ConvArgs& a) { return a.k == 3 && a.cin % 64 == 0 && a.cout % 64 == 0; }
bool wgrad_mfma_supported(const WgradArgs& a) { return a.cin % 32 == 0 && a.cout % 32 == 0; }
int64_t conv_mfma_splitk_floats(const ConvArgs& a) {
  const int64_t rows = (int64_t)a.n * a.hc * a.wc;
  return rows * a.cout < (1 << 22) ? 4 * rows * a.cout : 0;
}
bool thin_wgrad_mfma_supported(int ct, int cw, int wq, int dtype) { return dtype == 1 && ct <= 4 && cw % 16 == 0 && wq % 16 == 0; }
int64_t thin_wgrad_workspace_floats(int64_t q_pixels, int ct, int cw) { return (q_pixels / 256 + 1) * 9 * ct * cw; }
int64_t wgrad_mfma_workspace_floats(const WgradArgs& a) { return (int64_t)8 * a.cout * a.cin * a.k * a.k; }
int64_t wgrad_direct_workspace_floats(const WgradArgs& a) { return (int64_t)4 * a.cout * a.cin * a.k * a.k; }
int64_t thin_wgrad_mfma_workspace_floats(int n, int hq, int wq, int cw) { return ((int64_t)n * hq * wq / 1024 + 1) * 9 * 4 * cw; }
}  // namespace ae
