"""MI355X-native batched DLRM-style inference (SLS embedding bags, FC stacks,
pairwise-dot interaction).  ``rec`` binds the C-ABI library; ``synth`` holds
the seeded input generators and imports nothing else from this package."""
