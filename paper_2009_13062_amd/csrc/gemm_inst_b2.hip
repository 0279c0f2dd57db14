// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 2
// (8 = dense B with 16-byte aligned rows; 1 = dense B with any rows; 2 = strided pointwise convolution; 0 = implicit im2col B of a convolution).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<2>(int, int, GemmLaunch&, hipStream_t);
}
