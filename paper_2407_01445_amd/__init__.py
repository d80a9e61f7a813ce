"""MI355X-native FCCO global-contrastive-loss step (FastCLIP v0-v3): C-ABI library + binding.

Nothing heavy is imported here; `paper_2407_01445_amd.binding` loads the HIP library
and `paper_2407_01445_amd.workloads` holds the seeded input recipes.
"""
