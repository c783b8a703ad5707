// The hand-scheduled key-side backward kernel with the backward of the QK-norm (RMSNorm with gain, Sec.
// "Semi-Lipschitz control") in its epilogue: the same source, built to return the gradients with respect to the
// rows as they were before the normalisation, and a partial row of the gain gradient per workgroup.
#define TVM_PIPE_QKNORM 1
#include "bwd_col_pipe.hip"
