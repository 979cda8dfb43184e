#include "fa_launch.h"
namespace fa {
int launch_fwd_fp8(const void*, const void*, const void*, const float*, const float*, const float*, void*, float*, int, int, int, int, float, int, hipStream_t) { return FA_ERR_UNSUPPORTED; }
int launch_quant_hadamard(const void*, int, void*, float*, int, int, int, int, const signed char*, int, hipStream_t) { return FA_ERR_UNSUPPORTED; }
size_t bwd_workspace_bytes(int, int, int, int) { return 0; }
int launch_bwd(const void*, const void*, const void*, const void*, const float*, const void*, void*, void*, void*, void*, int, int, int, int, float, int, int, hipStream_t) { return FA_ERR_UNSUPPORTED; }
}
