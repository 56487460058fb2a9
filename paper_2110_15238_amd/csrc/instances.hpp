// The per-architecture list of template instances the profiler searches over (Section 3.2.2):
// some tens of (workgroup tile, wave grid, K depth, stages) combinations per kernel family, chosen by the hardware rules
// the paper states, restated for a CDNA4 compute unit:
//   - within the register budget (512 VGPR+AGPR per lane at one wave per SIMD) prefer large wave
//     tiles, they raise the FLOP per LDS byte;
//   - 4 or 8 waves per workgroup (1 or 2 per SIMD of the 4-SIMD compute unit);
//   - small problems need small workgroup tiles so that at least 256 workgroups exist.
// Each instance is compiled once into the library; tuning only runs them.
#pragma once
#include <vector>

#include "b2b_dma_kernel.hpp"
#include "b2b_kernel.hpp"
#include "conv_halo_kernel.hpp"
#include "conv_smallc_kernel.hpp"
#include "b2b_chain_kernel.hpp"
#include "b2b_halo_kernel.hpp"
#include "fprop_dma_kernel.hpp"
#include "fprop_kernel.hpp"
#include "fprop_pp_kernel.hpp"

// The lists below are what survived a measurement: every tile shape tried during development was
// timed by bolt_tune on the workloads of Section 4 (the ResNet-50 layers at batch 32, the GEMM and
// convolution shapes of Tables 1-3, the large shapes); an instance stays if it came within 5 % of the
// winner of at least one of them, or if it is the only cover of a corner (the two smallest tiles,
// the largest non-ping-pong tile).
//
// X(BM, BN, BK, WAVES_M, WAVES_N): B stored row-major, transposed through registers
#define BOLT_FPROP_TILE_LIST(X, XMODE, WMODE) \
  X(256, 256, 64, 2, 4, XMODE, WMODE),        \
  X(256, 128, 64, 4, 2, XMODE, WMODE),        \
  X(128, 256, 64, 2, 4, XMODE, WMODE),        \
  X(128, 128, 64, 2, 2, XMODE, WMODE),        \
  X(128, 128, 32, 2, 2, XMODE, WMODE),        \
  X(256, 64, 64, 4, 1, XMODE, WMODE),         \
  X(64, 128, 64, 2, 2, XMODE, WMODE),         \
  X(64, 64, 64, 2, 2, XMODE, WMODE),          \
  X(32, 64, 64, 1, 2, XMODE, WMODE),          \
  X(64, 32, 64, 2, 1, XMODE, WMODE)

// X(BM, BN, BK, WAVES_M, WAVES_N, STAGES): direct-to-LDS multi-stage instances (K-contiguous operands)
#define BOLT_FPROP_DMA_TILE_LIST(X, XMODE) \
  X(256, 256, 64, 2, 4, 2, XMODE),         \
  X(256, 128, 64, 4, 2, 3, XMODE),         \
  X(128, 256, 64, 2, 4, 3, XMODE),         \
  X(128, 128, 64, 2, 2, 2, XMODE),         \
  X(128, 128, 64, 2, 2, 3, XMODE),         \
  X(256, 64, 64, 4, 2, 3, XMODE),          \
  X(128, 64, 64, 4, 1, 3, XMODE),          \
  X(128, 64, 64, 2, 2, 3, XMODE),          \
  X(64, 128, 64, 2, 2, 3, XMODE),          \
  X(64, 64, 64, 2, 2, 3, XMODE),           \
  X(64, 64, 64, 2, 1, 4, XMODE),           \
  X(32, 64, 64, 1, 2, 4, XMODE),           \
  X(64, 32, 64, 2, 1, 4, XMODE),           \
  X(128, 64, 64, 2, 2, 2, XMODE),          \
  X(64, 128, 64, 2, 2, 2, XMODE),          \
  X(128, 128, 32, 2, 2, 3, XMODE),         \
  X(64, 64, 64, 2, 2, 2, XMODE),           \
  X(128, 128, 64, 2, 4, 2, XMODE),         \
  X(128, 128, 64, 2, 4, 3, XMODE),         \
  X(128, 128, 64, 1, 4, 2, XMODE),         \
  X(128, 256, 32, 2, 4, 3, XMODE),         \
  X(256, 64, 64, 4, 2, 2, XMODE),          \
  X(128, 128, 64, 2, 4, 4, XMODE),         \
  X(256, 128, 32, 4, 2, 2, XMODE),         \
  X(256, 128, 32, 2, 4, 3, XMODE),         \
  X(128, 64, 32, 2, 2, 3, XMODE)

// Single-stage tiles: the whole reduction is one k-tile (K <= tile K), so one operand buffer is
// enough and several workgroups share a compute unit, which hides the load and store latencies
// of these short-lived workgroups.
#define BOLT_FPROP_DMA_1STAGE_TILE_LIST(X, XMODE) \
  X(128, 128, 64, 2, 2, 1, XMODE),                \
  X(128, 64, 64, 2, 2, 1, XMODE),                 \
  X(64, 128, 64, 2, 2, 1, XMODE),                 \
  X(64, 64, 64, 2, 2, 1, XMODE)

// Tiles with k-groups: tile M, N, K, waves M, N, stages, x mode, k-groups.
#define BOLT_FPROP_DMA_KG_TILE_LIST(X, XMODE) \
  X(64, 64, 64, 2, 2, 2, XMODE, 2),           \
  X(64, 64, 64, 2, 2, 3, XMODE, 2),           \
  X(64, 128, 64, 2, 2, 2, XMODE, 2),          \
  X(128, 64, 64, 2, 2, 2, XMODE, 2),          \
  X(128, 128, 64, 2, 2, 2, XMODE, 2),         \
  X(128, 64, 64, 2, 2, 3, XMODE, 2),          \
  X(64, 128, 64, 2, 2, 3, XMODE, 2)

// Row-major weights through the direct-to-LDS pipeline (transposing LDS reads): tile M, N, K, waves M, N, stages, k-groups.
#define BOLT_FPROP_DMA_KN_TILE_LIST(X) \
  X(256, 256, 64, 2, 4, 2, 1),         \
  X(256, 128, 64, 4, 2, 3, 1),         \
  X(128, 256, 64, 2, 4, 3, 1),         \
  X(128, 128, 64, 2, 2, 3, 1),         \
  X(128, 128, 64, 2, 4, 3, 1),         \
  X(256, 64, 64, 4, 2, 3, 1),          \
  X(128, 64, 64, 2, 2, 3, 1),          \
  X(64, 128, 64, 2, 2, 3, 1),          \
  X(64, 64, 64, 2, 2, 3, 1),           \
  X(64, 64, 64, 2, 2, 2, 1),           \
  X(32, 64, 64, 1, 2, 4, 1),           \
  X(64, 32, 64, 2, 1, 4, 1),           \
  X(64, 64, 64, 2, 2, 2, 2),           \
  X(64, 64, 64, 2, 2, 3, 2),           \
  X(64, 128, 64, 2, 2, 2, 2),          \
  X(128, 64, 64, 2, 2, 2, 2),          \
  X(128, 128, 64, 2, 2, 1, 1),         \
  X(128, 64, 64, 2, 2, 1, 1),          \
  X(64, 128, 64, 2, 2, 1, 1),          \
  X(64, 64, 64, 2, 2, 1, 1),           \
  X(128, 64, 32, 2, 2, 3, 1),          \
  X(128, 128, 32, 2, 2, 3, 1),         \
  X(256, 128, 32, 2, 4, 3, 1)

namespace bolt {
// Each function appends its instances in a fixed order; kernel_id is the index in the op's table.
void register_gemm_kn_instances(std::vector<FpropInstance>& v);
void register_gemm_nk_instances(std::vector<FpropInstance>& v);
void register_gemm_kn_dma_instances(std::vector<FpropInstance>& v);
void register_conv_instances(std::vector<FpropInstance>& v);
void register_conv_halo_instances(std::vector<FpropInstance>& v);
void register_conv_align2_instances(std::vector<FpropInstance>& v);
void register_conv_smallc_instances(std::vector<FpropInstance>& v);
void register_conv_nchw_out_instances(std::vector<FpropInstance>& v);
void register_b2b_gemm_instances(std::vector<B2bInstance>& v);
void register_b2b_conv_instances(std::vector<B2bInstance>& v);
void register_b2b_gemm_dma_instances(std::vector<B2bInstance>& v);
void register_b2b_gemm_dma_kn_instances(std::vector<B2bInstance>& v);
void register_b2b_conv_dma_instances(std::vector<B2bInstance>& v);
void register_b2b_conv_halo_instances(std::vector<B2bInstance>& v);
void register_gemm_chain_instances(std::vector<ChainInstance>& v);
void register_conv_chain_instances(std::vector<ChainInstance>& v);
}  // namespace bolt
