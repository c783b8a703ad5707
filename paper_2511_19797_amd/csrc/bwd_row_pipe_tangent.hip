// The hand-scheduled query-side backward kernel for calls without gO (the gradient of <gTO, tO> alone,
// Steps 1-6 of App. C by themselves): the same source, built with the products of G left out.
#define TVM_PIPE_TANGENT_ONLY 1
#include "bwd_row_pipe.hip"
