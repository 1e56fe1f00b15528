// e2eg_layer_transform: placeholder until the MFMA kernels land (argument checks only).
#include "common.h"

using namespace e2eg;

extern "C" size_t e2eg_layer_transform_workspace_bytes(int32_t mode, int32_t n, int32_t Fin,
                                                       int32_t Fout, int32_t dtype) {
    (void)mode; (void)n; (void)Fin; (void)Fout; (void)dtype;
    return kAlign;
}

extern "C" int32_t e2eg_layer_transform(int32_t mode, int32_t n, int32_t Fin, int32_t Fout,
                                        int32_t dtype, int32_t relu, const void* d_P,
                                        const void* d_W, void* d_H, const void* d_gH, void* d_gP,
                                        float* d_gW, void* ws, size_t ws_bytes, void* stream) {
    (void)mode; (void)n; (void)Fin; (void)Fout; (void)dtype; (void)relu; (void)d_P; (void)d_W;
    (void)d_H; (void)d_gH; (void)d_gP; (void)d_gW; (void)ws; (void)ws_bytes; (void)stream;
    return fail(E2EG_ERR_INVALID_ARG, "layer_transform: not built yet");
}
