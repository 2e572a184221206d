"""Plain fp64 CPU oracle for the StreamBP hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package: it exists so that tests, the smoke check and the bench's
``cpu_baseline`` leg have an independent statement of what the HIP kernels
must compute.  It shares no code with ``paper_2506_03077_amd``.

Modules
-------
layer    full-sequence forward + reverse-mode backward of one pre-norm decoder
         layer (the ordinary gradient that the chunked method reaches exactly,
         Sec. 3.1 Eq. 1 and Sec. 3.2.2).
head     LM head + objective (SFT, GRPO, DPO) forward/backward (Sec. 3.2.1).
attn     causal attention of a chunk of queries against the prefix keys and
         values, forward and backward (Sec. 3.2.2, partitioned attention and
         Property 3.1).
lora     the same layer with low-rank adapters on its projection matrices and
         the adapter gradients (App. D, experiment setup: rank-32 adapters for
         the largest model); the masks of attn / layer beyond plain causality
         (sliding window, padding in front) are options of those modules.
chunked  the paper's chunk loop itself, in fp64, step by step (Sec. 3.2.1 and
         3.2.2) - used to check that per-chunk partial gradients sum to the
         full gradient and that chunk size does not matter.

Pin status: every function is pinned by tests/test_oracle_*.py (finite
differences, brute-force scalar loops, closed forms, structural invariants).
The paper prints no worked gradient values, so there are no printed-number
pins; none of the functions is "parity unpinned".
"""
