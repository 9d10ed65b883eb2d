// placeholder until the MoBA kernels land
#include "common.h"
namespace rs {
size_t moba_select_ws_bytes(const rs_shape *, long, int) { return RS_WS_CTRL_BYTES; }
int moba_select_dispatch(const rs_shape *, const void *, const void *, long, int, int, int, float *, int32_t *,
                         char *, hipStream_t) { return RS_UNSUPPORTED; }
size_t prefill_ws_bytes(const rs_shape *, long, int, int) { return RS_WS_CTRL_BYTES; }
int prefill_dispatch(const rs_shape *, const void *, const void *, const void *, long, int, float, const int32_t *,
                     int, void *, float *, char *, hipStream_t) { return RS_UNSUPPORTED; }
size_t snapkv_ws_bytes(const rs_shape *, long, int) { return RS_WS_CTRL_BYTES; }
int snapkv_dispatch(const rs_shape *, const void *, const void *, const void *, long, int, int, int, float, void *,
                    void *, long, int32_t *, float *, char *, hipStream_t) { return RS_UNSUPPORTED; }
}  // namespace rs
