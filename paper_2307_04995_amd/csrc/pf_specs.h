// Catalogue of statically specialised chain structures ("specs").
//
// The planner lowers every chain to micro-programs; when the lowered structure equals one of the entries
// below, the kernel instantiated for that entry is launched instead of the generic interpreter.  Only the
// structure is fixed at compile time (step codes, operand kinds and slots, operand counts, core kind);
// immediates and shapes stay run-time arguments.  The same table is expanded on the host (for matching)
// and on the device (for instantiation), so the two cannot drift apart.
#pragma once
#include "pf_common.h"

#define PF_U(code, kind, slot) ((uint32_t)(pf::code) | ((uint32_t)(pf::kind) << 8) | ((uint32_t)(slot) << 16))
#define PF_L(...) __VA_ARGS__

// X(id, NF, NV, NT, CORE, GAMMA, BETA, PRO, EPI)
//   NF / NV / NT : number of full operands, broadcast operands, temporaries
//   GAMMA / BETA : broadcast slots of the core's affine parameters (-1: none)
#define PF_ROW_SPECS(X)                                                                                        \
    /* x + res + bias -> LayerNorm -> GELU(erf) */                                                             \
    X(1, 2, 3, 0, CORE_LAYERNORM, 1, 2,                                                                        \
      PF_L(PF_U(U_MOV, K_FULL, 0), PF_U(U_ADD, K_FULL, 1), PF_U(U_ADD, K_VEC, 0)),                             \
      PF_L(PF_U(U_GELU_ERF, K_NONE, 0)))                                                                       \
    /* x + bias + res -> LayerNorm */                                                                          \
    X(2, 2, 3, 0, CORE_LAYERNORM, 1, 2,                                                                        \
      PF_L(PF_U(U_MOV, K_FULL, 0), PF_U(U_ADD, K_VEC, 0), PF_U(U_ADD, K_FULL, 1)), PF_L())                     \
    /* softmax, with an optional positive scale and causal mask folded into the core */                                                                                            \
    X(5, 1, 0, 0, CORE_SOFTMAX, -1, -1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L())                                  \
    /* LayerNorm */                                                                                            \
    X(6, 1, 2, 0, CORE_LAYERNORM, 0, 1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L())                                  \
    /* x + res -> LayerNorm */                                                                                 \
    X(7, 2, 2, 0, CORE_LAYERNORM, 0, 1, PF_L(PF_U(U_MOV, K_FULL, 0), PF_U(U_ADD, K_FULL, 1)), PF_L())          \
    /* RMSNorm */                                                                                              \
    X(8, 1, 1, 0, CORE_RMSNORM, 0, -1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L())                                   \
    /* x + res -> RMSNorm */                                                                                   \
    X(9, 2, 1, 0, CORE_RMSNORM, 0, -1, PF_L(PF_U(U_MOV, K_FULL, 0), PF_U(U_ADD, K_FULL, 1)), PF_L())

// Group family (channels-last GroupNorm): X(id, NF, NV, NT, CORE, GAMMA, BETA, PRO, EPI)
#define PF_GROUP_SPECS(X)                                                                                      \
    /* GroupNorm -> SiLU */                                                                                    \
    X(1, 1, 2, 0, CORE_GROUPNORM, 0, 1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L(PF_U(U_SILU, K_NONE, 0)))           \
    /* GroupNorm */                                                                                            \
    X(2, 1, 2, 0, CORE_GROUPNORM, 0, 1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L())

// Transpose family
#define PF_PERM_SPECS(X)                                                                                       \
    /* (x + bias) * scale -> permute */                                                                        \
    X(1, 1, 1, 0, CORE_PERMUTE, -1, -1,                                                                        \
      PF_L(PF_U(U_MOV, K_FULL, 0), PF_U(U_ADD, K_VEC, 0), PF_U(U_MUL, K_IMM, 0)), PF_L())                      \
    /* permute */                                                                                              \
    X(2, 1, 0, 0, CORE_PERMUTE, -1, -1, PF_L(PF_U(U_MOV, K_FULL, 0)), PF_L())

namespace pf {

struct SpecDesc {
    int id, nf, nv, nt, core, gamma, beta;
    int n_pro;
    uint32_t pro[8];
    int n_epi;
    uint32_t epi[8];
};

}  // namespace pf
