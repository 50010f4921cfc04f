"""CPU float64 oracle for paged-KV decode / observation-append attention.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import, link or execute anything in this directory; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  The oracle shares
no code, tables, constants or helpers with the HIP path.

What it defines: the engine's batched attention step over a paged KV cache during
multi-turn rollout -- the decode step (one query token per trajectory, the
bandwidth-bound phase) and the prefill of a new observation chunk on top of the
cached history (the compute-bound phase); Section 3.1 "Stage Computation" names the
two phases, Section 6.1 (the inference worker's step-wise loop) says a batch of
requests takes one decode or prefill step at a time, and Section 7.1 says prefix
caching keeps the history's KV.  The paper prints no formula, value or error bound
for this step, so the result is the textbook softmax-attention definition and every
pin in the CPU tests comes from mathematics (closed forms, invariants, brute force,
a library routine on the special case it covers), not from the paper:
"parity unpinned by the paper" for all functions here in that sense.

`kv_write` defines the step that precedes attention, the scatter of the new tokens' K/V
rows into the paged cache (with the E4M3 page-scale rule of FP8 pools); its header states
the reading taken and its pins.
"""
