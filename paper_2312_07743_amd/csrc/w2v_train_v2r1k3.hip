// window kernel, rows of 2 x 1 floats per lane, more than 12 output rows per window
#define W2V_VW 2
#define W2V_R 1
#define W2V_KMODE 3
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v2r1k3
#include "w2v_train_inst.inc"
