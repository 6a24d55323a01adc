"""MI355X-native rollout hot path: paged KV arena, decode attention, fused
token log-prob / KL.  The compiled library is loaded on first use of
`paper_2410_15651_amd.binding`; importing the package itself touches no GPU
and no shared object, so the input generators in `workloads` can be used
anywhere."""

__all__ = ["binding", "workloads"]
