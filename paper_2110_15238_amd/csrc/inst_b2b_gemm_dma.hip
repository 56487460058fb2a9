// Multi-stage fused GEMM pairs with direct-to-LDS operand loads (weights stored [N][K]).
#include "instances.hpp"
namespace bolt {
// Multi-stage fused GEMM pair for reduction-contiguous weights (B as [N][K]): the only family whose
// first weight matrix does not have to fit in LDS (Table 1's 576 x 128 case).
#define BDG(BM, BK, NW, N0T, N1T, NS) BOLT_B2B_DMA_INSTANCE(BM, BK, NW, N0T, N1T, NS, 0)
void register_b2b_gemm_dma_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      BDG(128, 64, 4, 64, 128, 3), BDG(128, 64, 4, 64, 128, 2), BDG(128, 64, 4, 128, 64, 2), BDG(128, 64, 4, 128, 64, 3),
      BDG(128, 64, 4, 64, 64, 3),  BDG(128, 64, 4, 32, 128, 3), BDG(128, 64, 4, 64, 32, 3),  BDG(128, 64, 4, 128, 128, 2),
      BDG(128, 64, 4, 64, 256, 2), BDG(64, 64, 2, 64, 128, 3),  BDG(128, 64, 4, 32, 128, 2),
      BDG(64, 64, 2, 64, 32, 3),
  };
  for (const auto& t : table) v.push_back(t);
}
// The same family for row-major weights (B as [K][N]).
#define BDK(BM, BK, NW, N0T, N1T, NS) BOLT_B2B_DMA_KN_INSTANCE(BM, BK, NW, N0T, N1T, NS)
void register_b2b_gemm_dma_kn_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      BDK(128, 64, 4, 64, 128, 3), BDK(128, 64, 4, 64, 128, 2), BDK(128, 64, 4, 128, 64, 2), BDK(128, 64, 4, 128, 64, 3),
      BDK(128, 64, 4, 64, 64, 3),  BDK(128, 64, 4, 32, 128, 3), BDK(128, 64, 4, 64, 32, 3),  BDK(128, 64, 4, 128, 128, 2),
      BDK(128, 64, 4, 64, 256, 2), BDK(64, 64, 2, 64, 128, 3),  BDK(128, 64, 4, 32, 128, 2),
      BDK(64, 64, 2, 64, 32, 3),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
