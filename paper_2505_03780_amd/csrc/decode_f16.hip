// fp16 instances of the paged decode kernels: the same source as the bf16 ones with the element
// type switched (fp16 I/O is what the paper's CUDA comparison ran; section "Evaluation").
#define ATTN_DECODE_ELEM_F16
#include "decode_bf16.hip"
