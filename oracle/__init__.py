"""Plain CPU oracle (test infrastructure only; see lstm_oracle.py)."""
from .lstm_oracle import (blstm_stack_backward, blstm_stack_forward, blstm_stack_loss,
                          lstm_backward, lstm_forward, sigmoid)

__all__ = ["lstm_forward", "lstm_backward", "blstm_stack_forward", "blstm_stack_backward",
           "blstm_stack_loss", "sigmoid"]
