"""MI355X-native fused rollout + GAE fragment (C ABI in include/msrl.h).

`binding` loads the HIP library and mirrors its entry points; `synth` holds the
seeded synthetic inputs.  Neither imports the CPU oracle.
"""
