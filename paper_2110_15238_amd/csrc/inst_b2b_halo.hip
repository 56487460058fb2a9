// Fused (stride-1 "same" conv) -> (1x1 conv) instances on the halo main loop.
#include "instances.hpp"
namespace bolt {
// BH(BM, WAVES, N0 tile, N1 tile, STAGES, XI)
#define BH(BM, NW, N0T, N1T, NS, XI) BOLT_B2B_HALO_INSTANCE(BM, NW, N0T, N1T, NS, XI)
#define BHC(BM, NW, N0T, N1T, NS, XI) BOLT_B2B_HALO_CHUNKED_INSTANCE(BM, NW, N0T, N1T, NS, XI)
void register_b2b_conv_halo_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      BH(128, 4, 64, 256, 2, 2), BH(128, 4, 64, 256, 3, 2), BH(256, 8, 64, 256, 2, 1), BH(256, 8, 64, 256, 3, 1),
      BH(64, 2, 64, 256, 3, 2),  BH(128, 4, 64, 64, 3, 2),  BH(128, 4, 64, 128, 3, 2), BH(128, 4, 128, 128, 2, 2),
      BH(256, 8, 64, 64, 3, 1),  BH(128, 4, 64, 64, 2, 2),  BH(256, 8, 64, 64, 2, 1),  BH(64, 2, 64, 64, 3, 2), BH(256, 4, 64, 64, 2, 2),
  };
  for (const auto& t : table) v.push_back(t);
  // op1 in chunks of 64 columns (wide second ops): BHC(BM, WAVES, N0 tile, N1 tile, STAGES, XI)
  static const B2bInstance chunked[] = {
      BHC(256, 4, 64, 256, 2, 2), BHC(128, 4, 64, 256, 2, 2), BHC(256, 8, 64, 256, 2, 1), BHC(256, 4, 64, 128, 2, 2),
  };
  for (const auto& t : chunked) v.push_back(t);
}
}  // namespace bolt
