// Internal interface between the DNN update and the NG-SGD preconditioner.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mavg {

// One layer's preconditioned weight/bias update for k replicas (replica = batch index).
struct NgLayerArgs {
    const int* dims; int L, l;                         // the network's widths d_0..d_L and this layer's index (1-based)
    int k, n, d_in, d_out;
    const float* A_in; int64_t a_ld, a_bstride;        // n x d_in input activations
    float* delta; int64_t ldd, d_bstride;              // n x d_out output derivatives (overwritten)
    float* W; float* b; int64_t theta_stride;          // d_out x d_in weights, d_out biases
    char* state_in; char* state_out; int64_t state_rstride;   // replica r's states at + r*state_rstride bytes
    int rank; float alpha, eta, lr;
    int mode;                                           // 0 apply only, 1 apply + fold, 2 first minibatch (three folds first)
    float* ws; int64_t ws_floats;
    float* gemm_ws; int64_t gemm_ws_floats;
};

// float32 elements of scratch ng_layer_update needs for the widest layer of the network
int64_t ng_dnn_ws_floats(const int* d, int L, int n, int k, int rank);
// returns 0 or a hipError_t.  Preconditions the two factors and applies the update; the folds of the states are
// left pending (their Y matrices stay in the scratch) until ng_dnn_finish.
int ng_layer_update(const NgLayerArgs& a, hipStream_t s);
// The same for all layers of the network at once (layers[l - 1] describes layer l; all share k, n, rank, alpha, eta,
// ws): one launch per step of the recipe instead of one per step and layer side.  Modes 0 and 1; in mode 1 the folds
// of all 2*L*k states (state (r, j) at ng_state + (r*2L + j)*state_stride bytes) are finished too, on an internal
// stream beside the weight update when one is available, and joined into `s` before the call's work is complete.
int ng_dnn_update(const NgLayerArgs* layers, int L, char* ng_state, int64_t state_stride, hipStream_t s);
// Fold this minibatch into all 2*L*k states (after ng_layer_update has run for every layer).
int ng_dnn_finish(const int* d, int L, int n, int k, int rank, float eta, char* ng_state, int64_t state_stride, float* ws,
                  hipStream_t s);

}  // namespace mavg
