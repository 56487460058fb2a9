// Persistent weights-resident back-to-back GEMM instances (row-major weights).
#include "instances.hpp"
namespace bolt {
#define SB(BM, BK, NW, N0T, N1T, NS) BOLT_STREAM_INSTANCE(BM, BK, NW, N0T, N1T, NS, 0, 1)
void register_b2b_gemm_stream_instances(std::vector<B2bInstance>& v) {
  static const B2bInstance table[] = {
      SB(64, 64, 2, 64, 128, 4), SB(128, 64, 4, 64, 128, 3), SB(128, 64, 4, 64, 32, 3), SB(128, 64, 4, 128, 64, 2),
      SB(128, 64, 4, 32, 128, 3),
  };
  for (const auto& t : table) v.push_back(t);
}
}  // namespace bolt
