// Three-op persistent chains (b2b_chain_kernel.hpp): compiled upper bounds (N0T, N1T, N2T) of the three
// output widths, for a GEMM first op (XMODE 0, weights stored [N][K] or row-major) and a convolution first op (XMODE 1).
#include "b2b_chain_kernel.hpp"
#include "instances.hpp"
namespace bolt {
// X(N0T, N1T, N2T, STAGES)
#define BOLT_CHAIN_WIDTHS(X, XMODE)                                                                          \
  X(64, 64, 64, 2, XMODE), X(64, 64, 64, 3, XMODE), X(64, 64, 128, 3, XMODE), X(64, 128, 64, 3, XMODE),       \
  X(64, 64, 256, 2, XMODE), X(64, 256, 64, 2, XMODE), X(128, 64, 64, 2, XMODE), X(128, 64, 128, 2, XMODE),     \
  X(64, 128, 128, 2, XMODE), X(128, 128, 64, 2, XMODE), X(128, 128, 128, 2, XMODE), X(32, 128, 32, 2, XMODE)
#define CH(N0T, N1T, N2T, NS, XMODE) BOLT_B2B_CHAIN_INSTANCE(128, 64, 4, N0T, N1T, N2T, NS, XMODE)
#define CHK(N0T, N1T, N2T, NS, XMODE) BOLT_B2B_CHAIN_KN_INSTANCE(128, 64, 4, N0T, N1T, N2T, NS)
void register_gemm_chain_instances(std::vector<ChainInstance>& v) {
  static const ChainInstance table[] = {BOLT_CHAIN_WIDTHS(CH, 0), BOLT_CHAIN_WIDTHS(CHK, 0)};  // [N][K], then [K][N] weights
  for (const auto& t : table) v.push_back(t);
}
// CHH(BM, WAVES, N0T, N1T, N2T, STAGES, XI): first op on the halo main loop (stride-1 "same" filters, C % 64 == 0)
#define CHH(BM, NW, N0T, N1T, N2T, NS, XI) BOLT_B2B_CHAIN_HALO_INSTANCE(BM, NW, N0T, N1T, N2T, NS, XI)
void register_conv_chain_instances(std::vector<ChainInstance>& v) {
  static const ChainInstance table[] = {
      BOLT_CHAIN_WIDTHS(CH, 1),
      CHH(128, 4, 64, 64, 64, 2, 2),  CHH(128, 4, 64, 64, 64, 3, 2),  CHH(256, 4, 64, 64, 64, 2, 2),
      CHH(128, 4, 64, 64, 128, 2, 2), CHH(128, 4, 64, 128, 64, 2, 2), CHH(128, 4, 64, 64, 256, 2, 2),
      CHH(128, 4, 64, 128, 128, 2, 2), CHH(128, 4, 128, 64, 64, 2, 2), CHH(128, 4, 128, 128, 128, 2, 2),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
