// fp16 instances of the LDS-ring prefill kernel: the same source as the bf16 ones, with the element
// traits switched (fp16 I/O is what the paper's CUDA comparison ran; section "Evaluation").
#define ATTN_RING_ELEM_F16
#include "prefill_bf16_ring.hip"
