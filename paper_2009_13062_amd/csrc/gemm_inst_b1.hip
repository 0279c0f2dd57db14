// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 1
// (8/4/1 = dense B read 1 elements wide; 0 = implicit im2col B of a convolution).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<1>(int, int, GemmLaunch&, hipStream_t);
}
