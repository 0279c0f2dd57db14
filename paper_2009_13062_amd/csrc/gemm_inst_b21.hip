// Instantiation of the bf16 MFMA contraction kernels for B-loader kind 21
// (stride-2 pointwise convolution over an even width read as pixel pairs, 1 per load).
#include "gemm_inst.h"
namespace nf {
template nf_status launch_gemm_bkind<21>(int, int, GemmLaunch&, hipStream_t);
}
