// Counters of the host-only HIP stand-in (hip_stub.cpp).  Test infrastructure.
#pragma once
#ifdef __cplusplus
extern "C" {
#endif
typedef struct {
    int violations;
    int kernel_launches, graph_launches, captures, instantiations, execs_destroyed;
    int streams_created, events_created, masked_streams_destroyed, device_syncs;
    int empty_branches;              /* streams that joined a capture and launched nothing in it */
    int max_graph_nodes;
    int max_live_execs;              /* most graph executables alive at once */
    int max_live_side_branches;      /* most parallel branches (side streams with nodes) among the executables alive at once */
    int live_streams, live_events, live_graphs, live_execs;   /* at the time of the call */
} hipstub_stats;
const hipstub_stats *hipstub_get_stats(void);
const char *hipstub_violation(int i);
#ifdef __cplusplus
}
#endif
