// The fused inner-grouped decode-attention kernels built for a paged store: the same source as the kernels
// for the contiguous store, compiled with the page-table lookup in (one entry per 64-token tile, fetched a
// tile ahead).  Exports launch_attention_inner_paged and attention_inner_paged_waves_per_cu.
#define INNERQ_PAGED_STORE 1
#include "attention_inner.hip"
