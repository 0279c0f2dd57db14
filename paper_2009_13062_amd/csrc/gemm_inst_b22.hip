// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 22
// (stride-2 pointwise convolution read as pixel pairs, 2 per load).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<22>(int, int, GemmLaunch&, hipStream_t);
}
