// window kernel, rows of one chunk of 4 floats plus four single floats per lane (dimensions 321..512 that are
// not multiples of 4: the chunk lies inside every row, the single floats are range-checked one by one),
// 7 to 12 output rows per window (two passes)
#define W2V_VW 4
#define W2V_R 1
#define W2V_TAIL 4
#define W2V_KMODE 2
#define W2V_WHOLE_ROWS 0
#define W2V_ENTRY train_fn_v4r1t4k2
#include "w2v_train_inst.inc"
