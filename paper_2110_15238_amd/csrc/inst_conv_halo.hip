// Stride-1 "same" convolution instances that re-use the activation halo out of LDS.
#include "instances.hpp"
namespace bolt {
// H(BM, BN, WAVES_M, WAVES_N, STAGES, XI): XI = halo load instructions per wave per issue point
#define H(BM, BN, WM, WN, NS, XI) BOLT_CONV_HALO_INSTANCE(BM, BN, WM, WN, NS, XI)
#define HK(BM, BN, WM, WN, NS, XI, KG) BOLT_CONV_HALO_KG_INSTANCE(BM, BN, WM, WN, NS, XI, KG)
void register_conv_halo_instances(std::vector<FpropInstance>& v) {
  static const FpropInstance table[] = {
      H(128, 64, 4, 1, 3, 2), H(256, 64, 4, 1, 3, 2), H(256, 64, 4, 2, 3, 1), H(64, 64, 2, 2, 3, 1), H(128, 128, 2, 2, 3, 1),
      // k-groups over the 64-channel chunks: HK(..., STAGES, XI, KG)
      HK(64, 64, 2, 2, 2, 1, 2), HK(64, 64, 2, 2, 2, 1, 4), HK(64, 128, 2, 2, 2, 1, 2), HK(128, 128, 2, 2, 2, 1, 2),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
