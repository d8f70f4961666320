"""MI355X-native batched execution of dynamic dataflow graphs (TreeLSTM, MV-RNN,
variable-length LSTM): C-ABI library `libacrobat.so` plus a thin ctypes binding."""
from .binding import (  # noqa: F401
    AcrobatError, Context, Dfg, acrobat_drnn_schedule, acrobat_schedule_birnn, acrobat_schedule_seqs, acrobat_schedule_trees, acrobat_strerror, EXPORTS, lib, acrobat_op_desc,
    OK, EINVAL, ESTRUCT, ENOMEM, EHIP, ETIMEOUT, TDC_SEQUENTIAL, TDC_INSTANCE_FIBERS, TDC_FORK_JOIN,
)
