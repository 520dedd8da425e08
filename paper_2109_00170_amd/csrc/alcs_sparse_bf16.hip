// The resident 1x1 kernels with X, the residual and Y stored as bfloat16 (namespace
// alcs::bf16io), behind alcs_sparse_conv_bf16: see the head of alcs_sparse.hip.
#define ALCS_FUSED_EPILOGUE 1
#define ALCS_IO_BF16 1
#include "alcs_sparse.hip"
