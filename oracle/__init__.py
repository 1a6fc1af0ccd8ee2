"""CPU references written from the paper -- TEST INFRASTRUCTURE ONLY.

estimator_oracle.c / oracle.py   the Estimator as a plain global-event-queue simulation (Section 4.2)
planner_oracle.py                the greedy planner, one simulation per candidate (Section 4.3)
envelope_oracle.py               traffic envelope and per-model ratios handed to the tuner (Section 5)
profile_oracle.py                tail of a measured latency distribution as a profile entry (Section 8)

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import anything from this
package; the library and its Python binding never do, and share no code with it.
"""
