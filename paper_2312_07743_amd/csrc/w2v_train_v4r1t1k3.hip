// window kernel, rows of one chunk of 4 floats plus one single float per lane (dimensions 260..320 that are
// multiples of 4), more than 12 output rows per window
#define W2V_VW 4
#define W2V_R 1
#define W2V_TAIL 1
#define W2V_KMODE 3
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v4r1t1k3
#include "w2v_train_inst.inc"
