// Operator descriptors (App. B.1-B.3), their configuration spaces, and the decoder that turns
// a configuration into launch geometry, resource needs and the -D constants of a template.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "common.hpp"
#include "space.hpp"

struct opevo_op {
    int kind = OPEVO_MATMUL;
    int dtype = OPEVO_BF16;
    // GEMM view: C[batch][M][N] = sum_K A[batch][M][K] B[batch][K][N]
    int64_t batch = 1, M = 0, N = 0, K = 0;
    bool trans_a = false;   // BMM only: A stored as [batch][K][M] (OPEVO_BMM_TA)
    // conv only
    int64_t cin = 0, hin = 0, win = 0, hk = 0, wk = 0, stride = 1, pad = 0, hout = 0, wout = 0, nimg = 0;

    double flops() const { return 2.0 * double(batch) * double(M) * double(N) * double(K); }
    int64_t a_elems() const;
    int64_t b_elems() const;
    int64_t c_elems() const { return batch * M * N; }
    int elem_size() const { return dtype == OPEVO_F32 ? 4 : 2; }
};

namespace opevo {

struct Decoded {
    opevo_plan plan;
    std::string tmpl;      // template name: "gemm_scalar" or "gemm_mfma"
    std::string defines;   // space separated -D options
    std::string kernel_name;   // symbol of the instantiated kernel
    int64_t zero_bytes = 0;    // bytes of the output the host clears before every launch (split reduction), else 0
    // pre-pass before every launch: 0 none; 1 Conv2d: the kernel reads channels-last copies of both operands;
    // 2 MatMul: the kernel reads a copy of the second operand transposed to [N][K]
    int prepass = 0;
};

// OPEVO_OK (plan.status says valid/invalid) or OPEVO_E_ILLEGAL / OPEVO_E_ARG.
int decode(const opevo_op &op, int variant, const int32_t *cfg, Decoded &out);
int op_param_descs(const opevo_op &op, int variant, std::vector<opevo_param_desc> &descs);

}  // namespace opevo
