// window kernel, rows of 1 x 5 floats per lane, 7 to 12 output rows per window (two passes)
#define W2V_VW 1
#define W2V_R 5
#define W2V_KMODE 2
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v1r5k2
#include "w2v_train_inst.inc"
