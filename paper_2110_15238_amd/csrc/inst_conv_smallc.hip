// First-layer convolutions (at most 4 input channels, NHWC without channel padding or NCHW input) and last-layer
// convolutions (NCHW output).
#include "instances.hpp"
namespace bolt {
void register_conv_smallc_instances(std::vector<FpropInstance>& v) {
  // (k-steps of 32 = 4 (filter row, channel) planes each, stride along W); the shorter k loop first: the built-in
  // pick rule keeps the first of equally ranked instances
  static const FpropInstance table[] = {BOLT_CONV_SMALLC_INSTANCE(3, 2), BOLT_CONV_SMALLC_INSTANCE(6, 2),
                                        BOLT_CONV_SMALLC_INSTANCE(3, 1), BOLT_CONV_SMALLC_INSTANCE(6, 1)};
  for (const auto& t : table) v.push_back(t);
}
// Last layers: the layout transformation folded into the store (output [N][K][P][Q]); a few general tiles for the
// gather (x mode 1) and for 1x1 / stride 1 / unpadded filters (x mode 0, GEMM addressing).
void register_conv_nchw_out_instances(std::vector<FpropInstance>& v) {
#define NO(BM, BN, WM, WN, NS, XMODE) BOLT_FPROP_DMA_NCHW_INSTANCE(BM, BN, 64, WM, WN, NS, XMODE)
  static const FpropInstance table[] = {NO(128, 128, 2, 2, 3, 1), NO(128, 64, 2, 2, 3, 1), NO(64, 128, 2, 2, 3, 1), NO(64, 64, 2, 2, 3, 1),
                                        NO(128, 128, 2, 2, 3, 0), NO(128, 64, 2, 2, 3, 0), NO(64, 128, 2, 2, 3, 0), NO(64, 64, 2, 2, 3, 0)};
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
