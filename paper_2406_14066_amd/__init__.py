"""MI355X-native batched speculative-verification step (lookahead attention over a
paged KV cache + rejection sampling with bonus token), behind a C ABI.

``spec_verify`` (the ctypes binding) loads the HIP library on first use and raises
if it has not been built; ``workloads`` generates the seeded synthetic inputs."""

__all__ = ["spec_verify", "workloads"]
