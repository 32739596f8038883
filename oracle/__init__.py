"""CPU oracle (test infrastructure only).

`oracle.reference` wraps the plain fp64 C routines of `dense_oracle.c`;
`oracle.planner` is the reference group planner in pure Python integers;
`oracle.rows` states batch forming (gather, scatter, dynamic fp8 scales) in numpy;
`oracle.simulator` replays a period of requests through the handler (the placement objective).
Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library never does, and this package never imports it.
"""
