/*
 * rnn.h -- C ABI for the other recurrent cells of the MI355X (gfx950) library: single-gate RNN
 * (ReLU or tanh) and GRU, forward pass and full back-propagation through time.
 *
 * Section 2 of Appleyard, Kocisky & Blunsom (arXiv 1604.01946) states that the optimisations carry
 * over to other recurrent units; Section 2.1 that a GRU offers two groups of three matrices to
 * combine and a single-gate RNN none; Section 3.3 lists ReLU, tanh, LSTM and GRU units.  The paper
 * prints no equations for them.  This library computes
 *
 *     single gate:  h_t = act(W x_t + R h_{t-1} + b)          act = max(0, .) or tanh
 *     GRU:          r_t = sigma(W_r x_t + R_r h_{t-1} + b_r)
 *                   z_t = sigma(W_z x_t + R_z h_{t-1} + b_z)
 *                   n_t = tanh (W_n x_t + b_n + r_t o (R_n h_{t-1}))
 *                   h_t = (1 - z_t) o n_t + z_t o h_{t-1}
 *
 * with the gates stacked in the order r, z, n along every 3H axis, one bias vector per gate, and
 * layers stacked as Section 2.4 describes.  The reset gate multiplies the recurrent product, so the
 * three recurrent matrices run as one stacked product per step (the grouping of Section 2.1).
 *
 * What runs: with H = 128, 256 or 512 (H = 512: B <= 2048, single gate 512; H = 256: 4096 / 2048; H = 128: 8192) the
 * persistent kernels of lstm.h with the weights on chip for all T steps (Section 4) and the layers
 * as a wavefront inside one launch (2.4; as many layers per launch as L*H/8 workgroups fit the CUs,
 * deeper stacks as consecutive groups of layers): their 32-row tile per workgroup holds, for 8 hidden units,
 * r, z and the input and recurrent halves of n (GRU), or the one gate and three empty groups
 * (single gate); with H = 1024 (B <= 512; single gate 256) or H = 2048 (B <= 320; single gate 96) the one-layer persistent kernels
 * with the recurrent matrix spread over all CUs.  Every other shape runs on the rungs of the paper's ladder that do not depend on the
 * cell: the input products of a layer batched over all steps (Section 2.3), the gates grouped into
 * one recurrent product per step (2.1), one fused point-wise kernel per step (2.2.2).  Weight
 * gradients are large products after propagation (2.6) in both cases, on the library's MFMA GEMM
 * kernels.  Hidden sizes below 512 other than 128 and 256 run zero-padded to the next of 128, 256, 512,
 * sizes between 512 and 1024 padded to 1024, and sizes between 1024 and 2048 with few rows (GRU: up to 64, from 1472
 * on up to 128; single gate: up to 64, from 1536 on up to 96) padded to 2048, on those persistent kernels (same rule, same reasoning and same effect on the reserve and workspace
 * sizes as in lstm.h: a padded unit stays at h = 0 and receives zero gradients, so the result is that of
 * the given network).  RNN_NO_PERSISTENT=1 in the environment keeps every shape, as given, on the
 * step-by-step path.
 *
 * Conventions: as in lstm.h (fp32, row-major, device pointers owned by the caller and 16-byte
 * aligned, asynchronous on `stream`, LSTM_* status codes, validation before any GPU work).
 * G = gates * H with gates = 1 (RNN_CELL_RELU, RNN_CELL_TANH) or 3 (RNN_CELL_GRU).
 * W is layer 0's [G][I] followed by the [G][H] matrices of layers 1..L-1; R is [L][G][H]; b is [L][G].
 */
#ifndef RNN_MI355X_H
#define RNN_MI355X_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RNN_CELL_RELU 0
#define RNN_CELL_TANH 1
#define RNN_CELL_GRU  2

/* Bytes of the `reserve` / `workspace` buffers for a shape; 0 for an unknown cell or a non-positive dimension. */
size_t rnn_reserve_bytes(int cell, int L, int T, int B, int I, int H);
size_t rnn_workspace_bytes(int cell, int L, int T, int B, int I, int H);

/*
 * Forward pass.  x [T][B][I]; h0 [L][B][H] or NULL (zeros); W, R, b as above.
 * Writes y [T][B][H] (hidden states of the top layer), hT [L][B][H] (or NULL: not written) and
 * `reserve` (required; opaque; what rnn_backward needs: every layer's hidden states and, for the
 * GRU, r, z, n and R_n h_{t-1}).  `workspace` is scratch of at least rnn_workspace_bytes().
 * Returns LSTM_OK, LSTM_INVALID_ARG, LSTM_BUFFER_TOO_SMALL or LSTM_HIP_ERROR.
 */
int rnn_forward(int cell, int L, int T, int B, int I, int H,
                const float* x, const float* h0, const float* W, const float* R, const float* b,
                float* y, float* hT, void* reserve, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward pass for Loss = <dy, y> + <dhT, hT>.  Inputs: those of the forward call, the reserve
 * it wrote, dy [T][B][H], dhT [L][B][H] or NULL (zeros).  Writes dx [T][B][I] (or NULL: skipped),
 * dh0 [L][B][H] (or NULL), dW, dR, db (shapes of W, R, b; overwritten).  Same return values.
 */
int rnn_backward(int cell, int L, int T, int B, int I, int H,
                 const float* x, const float* h0, const float* W, const float* R, const void* reserve,
                 const float* dy, const float* dhT,
                 float* dx, float* dh0, float* dW, float* dR, float* db,
                 void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
