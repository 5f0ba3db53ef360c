"""MI355X-native prefill hot path of MOM (mini-sequence SwiGLU MLP, last-token LM head,
KV offload).  The compute lives in the HIP library under `csrc/`; `binding` marshals
arguments to its C ABI; `synth` makes the seeded synthetic inputs."""

__all__ = ["binding", "synth", "build"]
