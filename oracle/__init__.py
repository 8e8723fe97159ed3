"""Plain CPU oracle (test infrastructure only; see lstm_oracle.py)."""
from .lstm_oracle import (blstm_stack_backward, blstm_stack_forward, blstm_stack_loss,
                          lstm_backward, lstm_forward, sigmoid)

from .chunking_oracle import chunk_batch, chunk_table
from .output_oracle import adam_step, sgd_momentum_step, softmax_ce_backward, softmax_ce_forward
from .stream_oracle import lstm_stream_forward_backward, segment_lengths
from .mdlstm_oracle import DIRECTIONS, mdlstm4_backward, mdlstm4_forward, mdlstm_backward, mdlstm_forward

__all__ = ["lstm_stream_forward_backward", "segment_lengths", "softmax_ce_forward", "softmax_ce_backward", "sgd_momentum_step", "adam_step", "chunk_table", "chunk_batch", "mdlstm_forward", "mdlstm_backward", "mdlstm4_forward", "mdlstm4_backward", "DIRECTIONS", "lstm_forward", "lstm_backward", "blstm_stack_forward", "blstm_stack_backward",
           "blstm_stack_loss", "sigmoid"]
