// window kernel, rows of 2 x 1 floats per lane, 7 to 12 output rows per window (two passes)
#define W2V_VW 2
#define W2V_R 1
#define W2V_KMODE 2
#define W2V_WHOLE_ROWS 1
#define W2V_ENTRY train_fn_v2r1k2
#include "w2v_train_inst.inc"
