// The resident 1x1 kernels with the depthwise 3x3 layer as their staging step (namespace
// alcs::dwpw), behind alcs_dw_sparse_conv_fused: see the head of alcs_sparse.hip.
#define ALCS_FUSED_EPILOGUE 1
#define ALCS_DW_STAGE 1
#include "alcs_sparse.hip"
