// fp16 build of the register-staged prefill kernel: the same source as the bf16 one, with the element
// type, the MFMA opcode and the instance table switched by this macro.
#define ATTN_PREFILL_ELEM_F16
#include "prefill_bf16.hip"
