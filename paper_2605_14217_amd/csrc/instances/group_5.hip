// written by gen_instances.py: do not edit by hand
#include "../mfma_kernel.hpp"
#include "../mfma_wide_kernel.hpp"
#include "../valu_kernel.hpp"

template __global__ void preft::mfma_tile_kernel<1, 1, 4, 0, false, 3, false, false, 2>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<1, 1, 8, 0, false, 1, false, false, 4>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<1, 1, 8, 0, false, 2, true, false, 0>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<1, 1, 8, 0, false, 3, true, false, 2>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<1, 1, 8, 8, true, 1, false, false, 2>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<2, 2, 4, 0, false, 1, false, false, 0>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_kernel<4, 2, 4, 0, true, 1, false, false, 0>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_layers_kernel<1, 1, 8, 0, false, 0>(preft::ApplyArgs);
template __global__ void preft::mfma_tile_layers_kernel<1, 2, 4, 0, false, 0>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<1, 1, 8, 1, true, 1, false, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<2, 1, 4, 1, false, 2, false, true>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<2, 1, 4, 2, false, 1, false, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<2, 1, 8, 1, false, 1, false, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<4, 1, 4, 1, false, 2, false, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<4, 1, 4, 1, true, 1, false, true>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_kernel<8, 1, 4, 1, false, 1, false, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_layers_kernel<1, 1, 4, 2, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_layers_kernel<2, 2, 4, 1, false>(preft::ApplyArgs);
template __global__ void preft::mfma_wide_layers_kernel<8, 1, 8, 1, false>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<1, 2, 4, true, 1, 8>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<1, 4, 1, true, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<2, 2, 4, true, 1, 8>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<2, 4, 4, false, 3, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<3, 4, 4, false, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<4, 4, 2, false, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<5, 2, 2, true, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<6, 2, 2, true, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<7, 2, 2, true, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_kernel<8, 2, 2, true, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_layers_kernel<1, 4, 4, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_layers_kernel<3, 4, 2, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_layers_kernel<5, 2, 2, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_layers_kernel<7, 2, 1, 0>(preft::ApplyArgs);
template __global__ void preft::valu_tile_layers_kernel<8, 2, 4, 8>(preft::ApplyArgs);
