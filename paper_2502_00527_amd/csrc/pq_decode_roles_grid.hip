// The role-specialised attention kernel with one work-group per (KV head, sequence, chunk), for
// launches of few units and for pq_decode_partials: the instantiations of pq_decode_roles.hip
// with the other scheduling mode.
#define PQ_ROLES_BALANCED false
#define PQ_ROLES_LAUNCH launch_attention_roles_grid
#include "pq_decode_roles.hip"
