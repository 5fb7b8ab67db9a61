"""CPU oracle for the cascaded video-analytics hot path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct implementations of
every stage (letterbox, conv graph, decode, top-k, NMS, ROI compaction,
crop-resize, classifier tail, batch-size search, portion scheduling, the
run-time rules of the serving loop).  It shares
no code with the HIP path and must never be imported by the product package;
only tests, the smoke check and the benchmark's CPU-baseline leg use it.

The paper treats per-model execution as a black box (Sec. III-A step 4), so the
stages follow their textbook definitions; the two scheduling algorithms follow
the paper's Algorithm 1 (batch-size part) and Algorithm 2 step by step.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
brute force, closed forms or invariants, except
  * sched.cwd_lite  - parity unpinned against the paper (no worked example is
    printed); pinned only by invariants and exhaustive search on small cases;
  * sched.coral     - parity unpinned against the paper; pinned by a
    hand-computed two-pipeline example and a schedule validator;
  * runtime.*       - parity unpinned against the paper (burstiness, lazy
    dropping and the horizontal scaler are named there without a formula or an
    example); pinned by hand-computed cases in tests/test_oracle_runtime.py.
"""
