// placeholder until the coder kernels land
#include "kvc_internal.h"
#include "../../include/kvc.h"
namespace kvc {
int launch_coder_tables(int, int, int, int, int, const CoderArgs &, const CoderArgs &, hipStream_t) { return KVC_ERR_UNSUPPORTED; }
int launch_encode_section(int, int, int, const CoderArgs &, hipStream_t) { return KVC_ERR_UNSUPPORTED; }
int launch_decode_prepare(const CoderArgs &, hipStream_t) { return KVC_ERR_UNSUPPORTED; }
int launch_decode_section(int, int, int, const CoderArgs &, hipStream_t) { return KVC_ERR_UNSUPPORTED; }
}
