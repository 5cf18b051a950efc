// window kernel, rows of 4 x 1 floats per lane, fewer than 6 output rows per window
#define W2V_VW 4
#define W2V_R 1
#define W2V_KMODE 0
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v4r1k0
#include "w2v_train_inst.inc"
