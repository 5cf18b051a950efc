// window kernel, rows of 1 x 5 floats per lane, fewer than 6 output rows per window
#define W2V_VW 1
#define W2V_R 5
#define W2V_KMODE 0
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v1r5k0
#include "w2v_train_inst.inc"
