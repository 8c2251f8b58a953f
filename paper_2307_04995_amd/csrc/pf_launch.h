// Host-callable launchers of the kernel families (implemented in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include "pf_common.h"

namespace pf {

hipError_t launch_row_generic(int dtype, const ChainArgs& a, const RowGeom& g, int k, bool reduce_only, bool ragged,
                              dim3 grid, dim3 block, hipStream_t st);
hipError_t launch_row_stream(int dtype, const ChainArgs& a, bool ragged, dim3 grid, hipStream_t st);
bool row_static_available(int spec_id, int kc, int rpw, bool wave_rows, unsigned block_threads);
hipError_t launch_row_static(int spec_id, int dtype, const ChainArgs& a, const RowGeom& g, int k, dim3 grid, dim3 block,
                             hipStream_t st);
hipError_t launch_ew(int dtype, const ChainArgs& a, uint32_t total_vecs, uint32_t vecs_per_row, int k, bool ragged,
                     dim3 grid, hipStream_t st);
hipError_t launch_perm(int spec_id, int dtype, const ChainArgs& a, const PermGeom& g, int variant, int k, bool ragged, dim3 grid,
                       dim3 block, uint32_t lds, hipStream_t st);
// phase 0: fused (resident) kernel; 1: statistics launch; 2: normalisation launch
hipError_t launch_group(int phase, bool general, int spec_id, int dtype, const ChainArgs& a, const GroupGeom& g, int nv, uint32_t tiles,
                        dim3 grid, dim3 block, uint32_t lds, hipStream_t st);
hipError_t launch_attn_decode(int dtype, const AttnArgs& a, int variant, int nv, dim3 grid, hipStream_t st);
hipError_t launch_stencil(int dtype, const ChainArgs& a, const StencilGeom& g, int variant, int ks, uint32_t lds, dim3 grid, hipStream_t st);
hipError_t launch_pool(int dtype, const ChainArgs& a, const PoolGeom& g, int op, int nv, dim3 grid, hipStream_t st);
// kc: 16-byte vectors per lane (the normalised extent is at most 32 * kc); one of 1, 2, 4, 16, 32 (eight vectors per
// lane compile to 240 registers, twice what sixteen need, so that size is left out)
hipError_t launch_colnorm(int dtype, const ColArgs& a, int kc, bool rms, bool ragged, dim3 grid, hipStream_t st);
hipError_t launch_gather(int dtype, const GatherArgs& a, int k, dim3 grid, hipStream_t st);
int group_resident_blocks_per_cu(int spec_id, int dtype, int nv, int block_threads);
// whole-tensor storage conversion, 16-bit <-> fp32 (n elements)
hipError_t launch_cast(int src_dtype, int dst_dtype, const void* src, void* dst, uint64_t n, hipStream_t st);
hipError_t launch_copy_probe(const void* src, void* dst, uint64_t bytes, int variant, hipStream_t st);

}  // namespace pf
