// Diagnostic settings taken from the environment.  They are read once, at the first library call that needs
// one, and again after lstm_shutdown(): a setting cannot change between a size query, a forward call and the
// backward call that reads its reserve, and no launch path calls getenv.
#pragma once

namespace lstm {

struct Knobs {
  bool no_pad;               // LSTM_NO_PAD=1: hidden sizes run as given instead of zero-padded to a persistent kernel's
  bool gemm_staged;          // LSTM_GEMM_STAGED=1: register-staged GEMM kernel everywhere
  bool rnn_pp;               // RNN_PINGPONG=0: the GRU and the single-gate cells on the one-chain wide kernels instead of the alternating ones
  bool large_ksplit;         // LSTM_LARGE_KSPLIT=0: a single slice at H = 1024 backward on 64 workgroups instead of 256
  bool gemm_swap;            // LSTM_GEMM_SWAP=0: no exchange of the operands' roles in the large-tile GEMM
  bool large_pp;             // LSTM_LARGE_PP=0: the one-chain forward kernel at H = 2048 instead of the alternating one
  int micro;                 // LSTM_MICRO=0: no pass runs as one workgroup; =2: every shape those kernels take does
  bool tiny;                 // LSTM_TINY=0: a single sequence (B = 1) on the narrow kernels instead of the flag-in-data ones
  bool gemm_split;           // LSTM_GEMM_SPLIT=0: no K slices for a product's last partial round of tiles
  int spin_limit;            // LSTM_SPIN_LIMIT: polls before a persistent kernel's wait gives up
  bool full_fences;          // LSTM_FULL_FENCES=1: release/acquire fences per step instead of the flag protocol
  bool coop_launch;          // LSTM_COOP_LAUNCH=1: cooperative launches for the persistent kernels
  bool plain_launch;         // LSTM_PLAIN_LAUNCH=1: persistent launches are not chained through an event
  bool two_chains;           // LSTM_CHAINS=2: two batch chains per workgroup in the narrow persistent kernels
  int fwd_narrow;            // LSTM_FWD_NARROW: -1 unset, 0 never slices / wide kernel, 1 one slice on the narrow kernel
  int bwd_narrow;            // LSTM_BWD_NARROW: the same for the backward kernels
  bool no_large_persistent;  // LSTM_NO_LARGE_PERSISTENT=1: H = 1024 / 2048 on the step path
  bool no_wgrad_overlap;     // LSTM_NO_WGRAD_OVERLAP=1: weight gradients never on the side stream
  bool fwd_batched_input;    // LSTM_FWD_BATCHED_INPUT=1: layer 0's input product as one GEMM although I == H
  bool rnn_no_persistent;    // RNN_NO_PERSISTENT=1: GRU / single-gate cells step by step
  int step_mt;               // LSTM_STEP_MT: 0 unset, else 1, 2 or 4 (hidden units per workgroup / 4 of the forward step kernel)
  int splitk_min_h;          // LSTM_SPLITK_MIN_H: smallest hidden size that takes the split-K backward step kernel (0 unset)
  int pingpong;              // LSTM_PINGPONG: -1 unset, 0 off, 1 on (two batch halves alternating on the matrix cores)
};

const Knobs& knobs();
void reset_knobs();

}  // namespace lstm
