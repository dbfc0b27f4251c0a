"""MI355X-native per-block knowledge distillation (hand-written HIP behind a C ABI).

`paper_2012_03096_amd.workloads` describes blocks and draws seeded inputs (no GPU needed);
`paper_2012_03096_amd.binding` loads libpbkd.so and exposes the pbkd_* calls.
"""
