"""CPU oracle for batched rollout generation: TEST INFRASTRUCTURE, not the product.

A plain, slow, fp64 restatement of what the rollout path computes: the generation stage
(prefill, then autoregressive decoding until a termination criterion; paper section 2.1,
"Optimization Workflow") and the inference stage's single teacher-forced forward pass
(same section).  The paper delegates the transformer and the sampler to its serving
engines and defines neither, so the operators here follow their standard public
definitions; every such reading is listed in the design notes.

Only the tests, the smoke check and the benchmark's cpu-baseline leg may import this
package.  It shares no code with the HIP library and never imports it.
"""
