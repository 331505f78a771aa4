"""MI355X-native GFlowNet rollout + Trajectory-Balance gradient (hand-written HIP behind a C ABI).

`paper_2511_16592_amd.gfnx` is the thin binding over libgfnx_hip.so (loaded lazily, fails loudly when
the library is missing); `paper_2511_16592_amd.workloads` holds the seeded synthetic inputs.
"""
