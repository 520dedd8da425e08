// alcs_sparse_conv_fused: the kernels of alcs_sparse.hip compiled once more with the fused
// epilogue (shortcut addition, ReLU / ReLU6) switched on, in namespace alcs::fused.
#define ALCS_FUSED_EPILOGUE 1
#include "alcs_sparse.hip"
