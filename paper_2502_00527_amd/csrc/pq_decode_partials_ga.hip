// pq_decode_partials_kernel for the grouped angle quantizer (Section 3.2 as printed): the
// instantiations of pq_decode_partials.hip with the per-group table rebuild.
#define PQ_PARTIALS_GA true
#define PQ_PARTIALS_LAUNCH launch_attention_partials_ga
#include "pq_decode_partials.hip"
