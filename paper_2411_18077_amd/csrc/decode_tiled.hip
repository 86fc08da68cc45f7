#include "decode_common.h"
namespace minikv {
int launch_decode_tiled(const DecArgs &a, int G, int units, bool mfma, hipStream_t st) { return MINIKV_EUNSUPPORTED; }
}
