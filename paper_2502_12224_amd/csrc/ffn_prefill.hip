#include "common.h"
#include "ffn_internal.h"
namespace fate {
fate_status launch_ffn_mfma(hipStream_t, const fate_ffn_desc&, DecodeArgs, float*, void*) {
    FATE_FAIL(FATE_ESHAPE, "MFMA path not built yet");
}
}
