"""MI355X-native pipeline-stage library (decoder-block stack for co-located
training and serving).  The compute lives in liblemix_stage.so (HIP, gfx950);
`binding` marshals arguments to its C ABI, `synth_inputs` makes seeded inputs.
Nothing here falls back to a CPU path: loading the binding without the built
library raises."""

__all__ = ["binding", "synth_inputs", "build"]
