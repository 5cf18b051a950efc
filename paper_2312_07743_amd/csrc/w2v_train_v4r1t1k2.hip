// window kernel, rows of one chunk of 4 floats plus one single float per lane (dimensions 260..320 that are
// multiples of 4), 7 to 12 output rows per window (two passes)
#define W2V_VW 4
#define W2V_R 1
#define W2V_TAIL 1
#define W2V_KMODE 2
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v4r1t1k2
#include "w2v_train_inst.inc"
