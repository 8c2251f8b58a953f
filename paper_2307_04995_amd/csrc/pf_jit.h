// Plan-time specialisation of the kernel templates (see pf_jit.cpp).
#pragma once
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "pf_common.h"

namespace pf {

// Spec id reported for a kernel that was specialised when the plan was made.
constexpr int kSpecJit = 255;

// The structure of a chain as template arguments: operand counts, core, and the packed micro-programs
// (code | kind << 8 | slot << 16 per step).
struct JitSpec {
    int nf = 0, nv = 0, nt = 0, core = 0, gamma = -1, beta = -1;
    int flags = 0;  // StaticSpec FLAGS_
    std::vector<uint32_t> pro, epi;
};

// false when PF_JIT=0 or PF_NO_STATIC=1
bool jit_enabled();
// kernels compiled so far in this process (cache hits do not count)
uint64_t jit_compile_count();
uint64_t jit_disk_hits();  // kernels taken from PF_JIT_CACHE instead of being compiled

// Each returns the kernel for the current device, or nullptr (reason in *err) when it cannot be produced.
// log2_lanes: lanes of a wave that share one row (6 = the whole wave; less: several rows side by side)
hipFunction_t jit_row_kernel(int device, int dtype, int kc, int rpw, bool wave_rows, bool ragged, int max_threads, int log2_lanes,
                             const JitSpec& spec, std::string* err);
// the same with the launch's shape as compile-time constants
struct RowShapeConst {
    uint32_t n_inner, mask_si, core_mask, vec_plain_all, waves_per_row, rows_per_block;
    uint64_t rows;
};
hipFunction_t jit_row_kernel_const(int device, int dtype, int kc, int rpw, bool wave_rows, bool ragged, int max_threads, int log2_lanes,
                                   const JitSpec& spec, const RowShapeConst& sh, std::string* err);
hipFunction_t jit_row_reduce_kernel(int device, int dtype, int k, bool ragged, const JitSpec& spec, std::string* err);
hipFunction_t jit_row_stream_kernel(int device, int dtype, bool ragged, const JitSpec& spec, std::string* err);
hipFunction_t jit_ew_kernel(int device, int dtype, int k, bool ragged, const JitSpec& spec, std::string* err);

// transpose family: variant 0 rows (k vectors per lane), 1 LDS-staged rows, 2 register-transposed tiles
hipFunction_t jit_perm_kernel(int device, int dtype, int variant, int k, bool ragged, const JitSpec& spec, std::string* err);
// the rows variant with the geometry of one launch shape as compile-time constants (vec_numel / vec_period: element
// count and row period of each broadcast operand, PF_DEV_MAX_VEC entries)
hipFunction_t jit_perm_rows_const(int device, int dtype, int k, const JitSpec& spec, const PermGeom& g, const uint32_t* vec_numel,
                                  const uint32_t* vec_period, std::string* err);
// group family: phase 0 fused, 1 statistics, 2 normalisation
hipFunction_t jit_group_kernel(int device, int dtype, int nv, int phase, int general_parts, const JitSpec& spec, std::string* err);
// stencil family (depthwise 3 x 3 convolution)
// the one-launch variant (phase 0) with the launch's geometry as compile-time constants
hipFunction_t jit_group_kernel_const(int device, int dtype, int nv, int general_parts, const JitSpec& spec, const GroupGeom& g, uint32_t tiles,
                                     uint32_t grid, uint32_t threads, std::string* err);
hipFunction_t jit_stencil_kernel(int device, int dtype, int variant, int ks, bool ragged, const JitSpec& spec, std::string* err);
// workgroups of `block_threads` threads one compute unit holds at once
hipFunction_t jit_pool_kernel(int device, int dtype, int nv, int op, bool ragged, const JitSpec& spec, std::string* err);
int jit_blocks_per_cu(hipFunction_t fn, int block_threads, uint32_t lds_bytes = 0);
// bytes of per-lane scratch memory the compiled kernel uses (register spills); 0 when it keeps everything in registers
int jit_scratch_bytes(hipFunction_t fn);

// params: addresses of the kernel's arguments, in order; lds_bytes: dynamic LDS
hipError_t jit_launch(hipFunction_t fn, dim3 grid, dim3 block, uint32_t lds_bytes, void** params, hipStream_t st);

}  // namespace pf
