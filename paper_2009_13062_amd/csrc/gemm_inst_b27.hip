// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 27
// (stride-2 pointwise convolution from a 14-wide image to 7 output columns, one input row per task).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<27>(int, int, GemmLaunch&, hipStream_t);
}
