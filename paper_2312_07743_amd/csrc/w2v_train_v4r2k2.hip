// window kernel, rows of 4 x 2 floats per lane, 7 to 12 output rows per window (two passes)
#define W2V_VW 4
#define W2V_R 2
#define W2V_KMODE 2
#define W2V_WHOLE_ROWS 1
#define W2V_ENTRY train_fn_v4r2k2
#include "w2v_train_inst.inc"
