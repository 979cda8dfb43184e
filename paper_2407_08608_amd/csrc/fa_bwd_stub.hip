#include "fa_launch.h"
namespace fa {
size_t bwd_workspace_bytes(int, int, int, int) { return 0; }
int launch_bwd(const void*, const void*, const void*, const void*, const float*, const void*, void*, void*, void*, void*, int, int, int, int, float, int, int, hipStream_t) { return FA_ERR_UNSUPPORTED; }
}
