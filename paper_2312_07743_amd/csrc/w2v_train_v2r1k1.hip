// window kernel, rows of 2 x 1 floats per lane, exactly 6 output rows per window
#define W2V_VW 2
#define W2V_R 1
#define W2V_KMODE 1
#define W2V_WHOLE_ROWS 1
#define W2V_ENTRY train_fn_v2r1k1
#include "w2v_train_inst.inc"
