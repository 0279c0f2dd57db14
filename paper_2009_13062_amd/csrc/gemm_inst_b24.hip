// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 24
// (stride-2 pointwise convolution read as pixel pairs, 4 per load).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<24>(int, int, GemmLaunch&, hipStream_t);
}
