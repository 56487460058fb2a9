// GEMM instances, B stored row-major [K][N] (transposed on the way to LDS).
#include "instances.hpp"
namespace bolt {
void register_gemm_kn_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {BOLT_FPROP_TILE_LIST(BOLT_FPROP_INSTANCE, 0, 1)};
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
