// Training step: forward that keeps each layer's input, MSE loss, and the
// backward pass with weights re-streamed in reverse order (paper Sec. 3.3).
#include "sp_engine.h"

int sp_layer_forward_train(sp_engine* e, int, const unsigned char*, int, int) {
    return sp_fail(e, SP_ERR_STATE, "training path not built");
}
int sp_layer_backward(sp_engine* e, int, const unsigned char*, int, int) {
    return sp_fail(e, SP_ERR_STATE, "training path not built");
}
int sp_train_begin(sp_engine* e, const float*, int, int) { return sp_fail(e, SP_ERR_STATE, "training path not built"); }
int sp_train_loss(sp_engine* e, const float*, float*, int, int) { return sp_fail(e, SP_ERR_STATE, "training path not built"); }
int sp_train_end(sp_engine* e, float*, int, int) { return sp_fail(e, SP_ERR_STATE, "training path not built"); }
