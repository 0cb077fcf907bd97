"""MI355X-native rollout generation and log-prob scoring for the SAPO node loop.

`paper_2509_08721_amd.sapo` is the binding over the C-ABI library (HIP kernels);
`paper_2509_08721_amd.workloads` makes seeded synthetic inputs.  Nothing here
computes on the CPU: the binding raises if the HIP library is not built.
"""
