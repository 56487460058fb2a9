// First-layer convolutions (at most 4 input channels, NHWC without channel padding or NCHW input).
#include "instances.hpp"
namespace bolt {
void register_conv_smallc_instances(std::vector<FpropInstance>& v) {
  // (k-steps of 32 = 4 (filter row, channel) planes each, stride along W); the shorter k loop first: the built-in
  // pick rule keeps the first of equally ranked instances
  static const FpropInstance table[] = {BOLT_CONV_SMALLC_INSTANCE(3, 2), BOLT_CONV_SMALLC_INSTANCE(6, 2),
                                        BOLT_CONV_SMALLC_INSTANCE(3, 1), BOLT_CONV_SMALLC_INSTANCE(6, 1)};
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
